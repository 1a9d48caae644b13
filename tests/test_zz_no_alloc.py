"""etv_tree_verify_attention_static: the attention call for callers that cannot allocate (the split partials live
in a fixed device array inside the library).  Its output must equal the output of etv_tree_verify_attention with a
caller's workspace -- same kernels, same launch plan, so the same bits -- on two calls in a row, the second on a
smaller input that finds the first call's partials still in the array.  Collected last on purpose."""
import numpy as np
import pytest
import torch

from paper_2603_08088_amd import api, synth
from gpu_helpers import DevWorkload, gpu_attention
from helpers import random_tree

pytestmark = pytest.mark.gpu


def _workload(seed, B, T, P, n_nodes, paged):
    rng = np.random.default_rng(seed)
    parents = [random_tree(rng, n_nodes[b]) for b in range(B)]
    return synth.assemble("static_ws", rng, parents, P, Hq=8, Hkv=2, d=128, dtype="bf16", V=512, W=T, paged=paged,
                          T_max=T, with_logits=False, spare_blocks=3)


def _both(wl, kv_split):
    d = DevWorkload(wl)
    m = api.build_tree_mask(d.parent, d.n_nodes)
    dsc = api.attn_desc(d.q, d.kt, d.k_cache, d.block_table, d.P_max, kv_split=kv_split)
    need = api.tree_verify_attention_workspace_bytes(dsc)
    ref_out, ref_lse = gpu_attention(d, m["bitmask"], kv_split=kv_split)
    out = torch.full_like(d.q, 7.0)                       # poisoned: every element must be overwritten
    lse = torch.full((wl.B, wl.Hq, wl.T_max), 7.0, dtype=torch.float32, device=d.q.device)
    api.tree_verify_attention_static(d.q, d.k_cache, d.v_cache, d.prefix_len, d.kt, d.vt, m["bitmask"], d.n_nodes,
                                     out, lse, P_max=d.P_max, block_table=d.block_table, kv_split=kv_split)
    torch.cuda.synchronize()
    return need, out, lse, ref_out, ref_lse


def test_static_workspace_call_equals_the_workspace_call_twice_in_a_row():
    # first call: several splits per sequence, ragged prefixes and node counts, paged cache
    big = _workload(4100, 3, 60, [2048, 700, 1], [60, 33, 1], True)
    need, out, lse, ref_out, ref_lse = _both(big, 128)
    assert 256 < need <= api.ATTN_STATIC_WORKSPACE_BYTES       # the call really used the array
    assert torch.equal(out, ref_out) and torch.equal(lse, ref_lse)
    # second call, smaller in every dimension: fewer sequences, rows and splits; the array still holds the first
    # call's partials where this one does not write
    small = _workload(4101, 1, 16, [300], [11], False)
    need2, out2, lse2, ref_out2, ref_lse2 = _both(small, 64)
    assert 256 < need2 < need
    assert torch.equal(out2, ref_out2) and torch.equal(lse2, ref_lse2)
    # and the library-chosen split of the first shape again
    need3, out3, lse3, ref_out3, ref_lse3 = _both(big, 0)
    assert torch.equal(out3, ref_out3) and torch.equal(lse3, ref_lse3)


def test_static_workspace_call_refuses_shapes_beyond_its_array():
    wl = _workload(4102, 1, 16, [300], [16], False)
    d = DevWorkload(wl)
    m = api.build_tree_mask(d.parent, d.n_nodes)
    # a descriptor whose partials would need gigabytes (128 splits of 8 x 256 x 32 rows): refused before any launch
    dsc = api.AttnDesc(B=8, T_max=256, Hq=32, Hkv=8, d=128, dtype=api.BF16, block_size=0, max_blocks=0, num_blocks=0,
                       P_cap=8448, P_max=8192, scale=0.0, kv_split=64, flags=0)
    assert api.tree_verify_attention_workspace_bytes(dsc) > api.ATTN_STATIC_WORKSPACE_BYTES
    out = torch.full_like(d.q, 7.0)
    with pytest.raises(api.EtvError) as e:
        api.tree_verify_attention_static(d.q, d.k_cache, d.v_cache, d.prefix_len, d.kt, d.vt, m["bitmask"], d.n_nodes,
                                         out, None, P_max=8192, desc=dsc)
    assert e.value.rc == -3
    torch.cuda.synchronize()
    assert torch.all(out == 7.0)                           # nothing was launched


def test_static_workspace_call_inside_a_replayed_hip_graph():
    """What the entry point is for: captured once, replayed several times with new inputs in the same buffers and
    eager work in between; every replay must give the bits of an eager call with a workspace on the same inputs."""
    wl = _workload(4103, 2, 40, [900, 333], [40, 17], True)
    d = DevWorkload(wl)
    m = api.build_tree_mask(d.parent, d.n_nodes)
    out = torch.empty_like(d.q)
    lse = torch.empty((wl.B, wl.Hq, wl.T_max), dtype=torch.float32, device=d.q.device)

    def call():
        api.tree_verify_attention_static(d.q, d.k_cache, d.v_cache, d.prefix_len, d.kt, d.vt, m["bitmask"], d.n_nodes,
                                         out, lse, P_max=d.P_max, block_table=d.block_table, kv_split=128)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        call()                                            # first call on the device outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call()
    gen = torch.Generator(device="cuda").manual_seed(5)
    for rep in range(4):
        d.q.copy_(torch.randn(d.q.shape, generator=gen, device="cuda").to(torch.bfloat16))   # eager work between replays
        d.kt.copy_(torch.randn(d.kt.shape, generator=gen, device="cuda").to(torch.bfloat16))
        out.fill_(7.0)
        graph.replay()
        ref_out, ref_lse = gpu_attention(d, m["bitmask"], kv_split=128)
        torch.cuda.synchronize()
        assert torch.equal(out, ref_out) and torch.equal(lse, ref_lse), rep
