#!/usr/bin/env python3
"""Benchmark of the tree-verify step on one MI355X.

One step = one pass of the whole verification path over one batch of synthetic input:
  build_tree_mask -> tree_verify_attention for each of the model's layers -> safe_gather_paths ->
  evaluate_posterior -> commit_accepted_kv over all layers (one launch),
with every input already resident in HBM.  The step is captured once into a HIP graph per cache
set and replayed; cache sets are rotated so that consecutive steps stream K/V from HBM, not from
the 256 MB memory-side cache.  Prints ONE compact JSON line on stdout (metric: tree-verify tokens/s); --report FILE
writes the full report (plans, traffic, sample descriptions, every figure unrounded) as well ("-": to stderr).

The default workload is the largest single-GPU configuration: the T = 128, depth 10 cell of the budget sweep
(B = 32 sequences, 4096-token paged prefixes, 32 layers).  Beside the headline the line carries
  * `roofline`: the attention launch (the dominant kernel) against the published peaks and against what this
    machine sustains in the same run (a streaming-read probe and a register-only MFMA probe);
  * `timing`: median and minimum over >= 50 event-timed replays of the whole step and of each part of it;
  * `configs`: the attention launch at every configuration (C2, C3, C4 and the T = 8 ... 128 sweep cells), median and
    minimum over >= 50 timed samples, with both roofline fractions;
  * `cpu_baseline`: the CPU oracle timed on a bounded sample of the same workload and scaled to a step.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c2|c2_paged|c3|c4|c5_T<T>_D<D>[_B<B>_P<P>]] [--layers L]
                  [--no-graph] [--skip-cpu] [--no-configs] [--kv-split N]
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published peak
MFMA_BF16_PEAK_TFLOPS = 2500.0


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="c5_T128_D10")
    ap.add_argument("--layers", type=int, default=32)
    ap.add_argument("--no-graph", action="store_true")
    ap.add_argument("--skip-cpu", action="store_true")
    ap.add_argument("--kv-split", type=int, default=0)
    ap.add_argument("--attn-flags", type=int, default=0)
    ap.add_argument("--no-lm-head", action="store_true", help="skip the timing of the fused head + argmax kernel")
    ap.add_argument("--no-branch-cache", action="store_true",
                    help="skip the timing of branch replication and the commit by path indices")
    ap.add_argument("--calib-copy-mib", type=int, default=0,
                    help="also run one device copy of this many MiB (a known-size kernel to calibrate profiler byte counters)")
    ap.add_argument("--no-configs", action="store_true", help="skip the per-configuration table of attention launches")
    ap.add_argument("--samples", type=int, default=50, help="event-timed samples per figure (at least 50)")
    ap.add_argument("--no-probes", action="store_true", help="skip the stream-read and MFMA probes")
    ap.add_argument("--report", default="", help="also write the full report (JSON) to this file; '-' = one line on stderr")
    ap.add_argument("--sets", type=int, default=0, help="cache sets to rotate over (0 = enough to exceed 640 MB)")
    return ap.parse_args()


def make_host_workload(name, with_cache=False, with_logits=True):
    from paper_2603_08088_amd import synth
    kw = dict(with_cache=with_cache, with_logits=with_logits)
    if name == "c2":
        return synth.config2(**kw), "7B-class GQA verify step: B=1, 32/8 heads, d=128, bf16, P=2048, 60-node tree"
    if name == "c2_paged":
        return synth.config2(paged=True, **kw), "config 2 with a paged prefix cache"
    if name == "c3":
        return synth.config3(**kw), "ragged batch: B=8, P~U[512,8192], paged, 60-node trees"
    if name == "c4":
        return synth.config4(**kw), "long context: B=1, P=32768, 128-node tree"
    m = re.fullmatch(r"c5_T(\d+)_D(\d+)(?:_B(\d+)_P(\d+))?", name)
    if m:
        B, P = int(m.group(3) or 32), int(m.group(4) or 4096)
        return synth.config5(int(m.group(1)), int(m.group(2)), B=B, P=P, **kw), \
            f"budget sweep cell: B={B}, P={P} paged, T={m.group(1)}, depth {m.group(2)}, 32/8 heads, d=128, bf16"
    raise SystemExit(f"unknown workload {name}")


# the attention launch of every configuration (the sweep cells at the depth whose traffic counters are on file)
TABLE_CONFIGS = ("c2", "c3", "c4", "c5_T8_D4", "c5_T16_D10", "c5_T32_D6", "c5_T64_D8", "c5_T128_D10")


class Step:
    """Device state of one workload and the launch sequence of a step."""

    def __init__(self, wl, layers, nsets, kv_split, attn_flags=0):
        import numpy as np
        import torch
        from paper_2603_08088_amd import api
        from paper_2603_08088_amd.devio import to_dev
        self.api, self.torch, self.wl, self.L = api, torch, wl, layers
        dev = "cuda:0"
        gen = torch.Generator(device=dev)
        gen.manual_seed(26030808)
        B, T, Hq, Hkv, d = wl.B, wl.T_max, wl.Hq, wl.Hkv, wl.d
        self.parent, self.n_nodes = to_dev(wl.parent), to_dev(wl.n_nodes)
        self.tokens, self.retrieve = to_dev(wl.tokens), to_dev(wl.retrieve)
        self.prefix_len, self.capacity = to_dev(wl.prefix_len), to_dev(wl.capacity)
        self.block_table = to_dev(wl.block_table)
        self.logits = to_dev(wl.logits)
        self.P_max = int(wl.prefix_len.max())
        bf = torch.bfloat16

        def rnd(*shape):
            return torch.randn(shape, generator=gen, device=dev, dtype=torch.float32).to(bf)
        self.q = rnd(layers, B, T, Hq, d)
        self.kt, self.vt = rnd(layers, B, T, Hkv, d), rnd(layers, B, T, Hkv, d)
        cshape = (wl.num_blocks, Hkv, 16, d) if wl.paged else (B, wl.P_cap, Hkv, d)
        per_set = 2 * layers * int(np.prod(cshape)) * 2
        self.nsets = nsets if nsets > 0 else max(1, -(-640 * 2 ** 20 // per_set))
        self.kc = [torch.empty((layers,) + cshape, dtype=bf, device=dev) for _ in range(self.nsets)]
        self.vc = [torch.empty((layers,) + cshape, dtype=bf, device=dev) for _ in range(self.nsets)]
        for s in range(self.nsets):
            for l in range(layers):   # layer by layer keeps the fp32 staging buffer small
                self.kc[s][l].copy_(torch.randn(cshape, generator=gen, device=dev, dtype=torch.float32))
                self.vc[s][l].copy_(torch.randn(cshape, generator=gen, device=dev, dtype=torch.float32))
        self.cache_bytes = per_set * self.nsets
        # outputs and workspaces, allocated once
        i32 = dict(dtype=torch.int32, device=dev)
        words = (T + 63) // 64
        L_max, W = wl.retrieve.shape[1], wl.W
        # the tree tensors of a step are built on the device from `parent` (mask, depth, position ids, path table);
        # the host-built path table of the workload is only used to check the device one once, before timing
        self.L_max, self.W = L_max, W
        self.mask_out = dict(bitmask=torch.empty((B, T, words), dtype=torch.int64, device=dev),
                             dense=torch.empty((B, 1, T, T), dtype=torch.uint8, device=dev),
                             depth=torch.empty((B, T), **i32), status=torch.empty((B,), **i32),
                             position_ids=torch.empty((B, T), **i32), retrieve=torch.empty((B, L_max, W), **i32),
                             n_paths=torch.empty((B,), **i32))
        api.tensorize_tree(self.parent, self.n_nodes, self.prefix_len, L_max, W, out=self.mask_out)
        torch.cuda.synchronize()
        assert torch.equal(self.mask_out["retrieve"], self.retrieve), "device path table differs from the workload's"
        self.retrieve = self.mask_out["retrieve"]
        self.out = torch.empty((layers, B, T, Hq, d), dtype=bf, device=dev)
        self.desc = api.attn_desc(self.q[0], self.kt[0], self.kc[0][0], self.block_table, self.P_max, 0.0, kv_split, attn_flags)
        self.ws = torch.empty((max(256, api.tree_verify_attention_workspace_bytes(self.desc)),), dtype=torch.uint8,
                              device=dev)
        self.tokens3 = self.tokens.reshape(B, T, 1)
        self.gather_out = dict(safe=torch.empty((B, L_max, W), **i32),
                               pvalid=torch.empty((B, L_max, W), dtype=torch.uint8, device=dev),
                               gathered=torch.empty((B, L_max, W, 1), **i32))
        self.post_out = dict(argmax=torch.empty((B, T), **i32), len=torch.empty((B, L_max), **i32),
                             best=torch.empty((B,), **i32), accept_len=torch.empty((B,), **i32),
                             acc_nodes=torch.empty((B, W), **i32), bonus=torch.empty((B,), **i32))
        self.post_ws = torch.empty((max(256, api.evaluate_posterior_workspace_bytes(B, T, wl.V)),),
                                   dtype=torch.uint8, device=dev)
        self.commit_out = dict(prefix_len_out=torch.empty((B,), **i32), slot_map=torch.empty((B, W), **i32),
                               status=torch.empty((B,), **i32))

    def attention_layers(self, s):
        api = self.api
        for l in range(self.L):
            api.tree_verify_attention(self.q[l], self.kc[s][l], self.vc[s][l], self.prefix_len, self.kt[l],
                                      self.vt[l], self.mask_out["bitmask"], self.n_nodes, P_max=self.P_max,
                                      block_table=self.block_table, out=self.out[l], want_lse=False,
                                      workspace=self.ws, desc=self.desc)

    def run(self, s):
        api = self.api
        api.tensorize_tree(self.parent, self.n_nodes, self.prefix_len, self.L_max, self.W, out=self.mask_out)
        self.attention_layers(s)
        self.epilogue(s)

    def epilogue(self, s):
        # gather + acceptance + commit as the fused epilogue; the new prefix length goes to its own buffer so that
        # every timed step sees the same prefix
        api = self.api
        api.verify_epilogue(self.logits, self.tokens, self.retrieve, self.n_nodes, self.kt, self.vt, self.kc[s],
                            self.vc[s], self.prefix_len, self.capacity, block_table=self.block_table, dummy=0,
                            src=self.tokens3, workspace=self.post_ws, gather_out=self.gather_out,
                            post_out=self.post_out, commit_out=self.commit_out)

    def capture(self, fn):
        return capture(self.torch, fn)


def attention_algorithmic(wl):
    """Algorithmic bytes and flops of one attention launch (one layer): prefix K/V read once, tree K/V,
    Q read and O written; 4*Hq*T*(P+T)*d flops."""
    e = 2 if wl.dtype == "bf16" else 4
    by = fl = 0
    for b in range(wl.B):
        P, T = int(wl.prefix_len[b]), int(wl.n_nodes[b])
        by += 2 * P * wl.Hkv * wl.d * e + 2 * T * wl.Hkv * wl.d * e + 2 * T * wl.Hq * wl.d * e
        fl += 4 * wl.Hq * T * (P + T) * wl.d
    return by, fl


def event_samples(torch, fn, n, warm=5):
    """Milliseconds of n calls of fn, each between its own pair of HIP events on the launch stream."""
    for i in range(warm):
        fn(i)
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
    ev[0].record()
    for i in range(n):
        fn(warm + i)
        ev[i + 1].record()
    torch.cuda.synchronize()
    return [ev[i].elapsed_time(ev[i + 1]) for i in range(n)]


def stats_us(samples_ms, per=1):
    import statistics
    us = [x * 1e3 / per for x in samples_ms]
    return {"median_us": statistics.median(us), "min_us": min(us), "mean_us": sum(us) / len(us), "samples": len(us)}


def traffic_on_file(name):
    """HBM bytes per attention launch from the rocprofv3 counter runs kept under profiles/ (None if not taken)."""
    tpath = os.path.join(ROOT, "profiles", f"attention_hbm_traffic_{name}.txt")
    if os.path.exists(tpath):
        return json.load(open(tpath)).get("hbm_bytes_per_launch")
    return None


def fractions(by, fl, us, peaks):
    """Both roofline fractions of a launch of `us` microseconds, against the published and the measured ceilings."""
    gbs, tfl = by / (us * 1e-6) / 1e9, fl / (us * 1e-6) / 1e12
    out = {"hbm_gbs": gbs, "mfma_tflops": tfl, "hbm_frac": gbs / HBM_PEAK_GBS, "mfma_frac": tfl / MFMA_BF16_PEAK_TFLOPS,
           "bound": "hbm" if by / HBM_PEAK_GBS / 1e9 >= fl / MFMA_BF16_PEAK_TFLOPS / 1e12 else "mfma"}
    if peaks.get("stream_gbs"):
        out["hbm_frac_of_measured"] = gbs / peaks["stream_gbs"]
    if peaks.get("mfma_sustained_tflops"):
        out["mfma_frac_of_measured"] = tfl / peaks["mfma_sustained_tflops"]
    return out


def run_probes(torch):
    """What this machine sustains, measured in the same run: a 1 GiB streaming read, and a register-only MFMA loop
    on every compute unit, first launch and sustained (the chip lowers its clock under matrix load)."""
    from paper_2603_08088_amd import probe
    buf = torch.empty(2 ** 30, dtype=torch.uint8, device="cuda:0").fill_(1)
    sink = torch.zeros(16, dtype=torch.uint8, device="cuda:0")
    ms = event_samples(torch, lambda i: probe.hbm_read_probe(buf, sink), 10, warm=2)
    stream_gbs = buf.numel() / (min(ms) * 1e-3) / 1e9
    stream_gbs_median = buf.numel() / (sorted(ms)[len(ms) // 2] * 1e-3) / 1e9
    del buf
    torch.cuda.synchronize()
    time.sleep(0.5)                       # let the clocks recover so that the first launch is a cold one
    iters = 128                           # ~0.55 TFLOP per launch: a few hundred microseconds, like an attention launch
    fl = probe.mfma_bf16_probe_flops(iters)
    ms = event_samples(torch, lambda i: probe.mfma_bf16_probe(iters, sink), 200, warm=0)
    tail = sorted(ms[100:])
    # the matrix instructions of the headline attention launch (66 tiles of 64 keys, 32 rows per wavefront, 512
    # workgroups) on operands that change from product to product, nothing else in the kernel
    lfl = probe.mfma_bf16_live_probe_flops(66)
    lms = sorted(event_samples(torch, lambda i: probe.mfma_bf16_live_probe(66, sink), 100, warm=20))
    return {"stream_gbs": stream_gbs, "stream_gbs_median": stream_gbs_median,
            "mfma_attention_products_tflops": lfl / (lms[len(lms) // 2] * 1e-3) / 1e12,
            "mfma_first_launch_tflops": fl / (ms[0] * 1e-3) / 1e12,
            "mfma_best_launch_tflops": fl / (min(ms) * 1e-3) / 1e12,
            "mfma_sustained_tflops": fl / (tail[len(tail) // 2] * 1e-3) / 1e12,
            "mfma_probe": f"200 back-to-back launches of {fl / 1e12:.2f} TFLOP (v_mfma_f32_32x32x16_bf16 from registers, "
                          "2048 workgroups x 4 wavefronts); sustained = median of launches 101-200"}


class AttnOnly:
    """Attention launches of one configuration over enough layers of cache (at least eight, at least 640 MB) that
    K/V streams from HBM."""

    def __init__(self, name, torch, api):
        from paper_2603_08088_amd.devio import to_dev
        wl, self.text = make_host_workload(name, with_logits=False)
        self.wl, self.api, self.torch = wl, api, torch
        dev, bf = "cuda:0", torch.bfloat16
        gen = torch.Generator(device=dev)
        gen.manual_seed(26030808)
        B, T, Hq, Hkv, d = wl.B, wl.T_max, wl.Hq, wl.Hkv, wl.d
        cshape = (wl.num_blocks, Hkv, 16, d) if wl.paged else (B, wl.P_cap, Hkv, d)
        per_layer = 2 * 2
        for x in cshape:
            per_layer *= x
        # at least eight launches per sample: a graph replay costs several microseconds of its own, which two
        # launches of 90 us would each carry half of
        self.layers = max(8, -(-640 * 2 ** 20 // per_layer))
        L = self.layers
        self.q = torch.randn((L, B, T, Hq, d), generator=gen, device=dev).to(bf)
        self.kt = torch.randn((L, B, T, Hkv, d), generator=gen, device=dev).to(bf)
        self.vt = torch.randn((L, B, T, Hkv, d), generator=gen, device=dev).to(bf)
        self.kc = torch.empty((L,) + cshape, dtype=bf, device=dev)
        self.vc = torch.empty((L,) + cshape, dtype=bf, device=dev)
        for l in range(L):
            self.kc[l].copy_(torch.randn(cshape, generator=gen, device=dev))
            self.vc[l].copy_(torch.randn(cshape, generator=gen, device=dev))
        self.out = torch.empty_like(self.q)
        self.parent, self.n_nodes = to_dev(wl.parent), to_dev(wl.n_nodes)
        self.prefix_len, self.block_table = to_dev(wl.prefix_len), to_dev(wl.block_table)
        self.P_max = int(wl.prefix_len.max())
        self.bitmask = api.build_tree_mask(self.parent, self.n_nodes, want_dense=False, want_depth=False)["bitmask"]
        self.desc = api.attn_desc(self.q[0], self.kt[0], self.kc[0], self.block_table, self.P_max)
        self.ws = torch.empty((max(256, api.tree_verify_attention_workspace_bytes(self.desc)),), dtype=torch.uint8,
                              device=dev)

    def launches(self):
        for l in range(self.layers):
            self.api.tree_verify_attention(self.q[l], self.kc[l], self.vc[l], self.prefix_len, self.kt[l], self.vt[l],
                                           self.bitmask, self.n_nodes, P_max=self.P_max, block_table=self.block_table,
                                           out=self.out[l], want_lse=False, workspace=self.ws, desc=self.desc)


def capture(torch, fn):
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        fn()                      # warm up outside capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    with torch.cuda.graph(g):
        fn()
    return g


def configs_table(torch, api, n_samples, peaks, headline=None):
    """The attention launch at every configuration: a sample is one replay of a graph of `layers` launches over
    distinct layer caches (so K/V comes from HBM); median and minimum over the samples, per launch."""
    rows = {}
    for name in TABLE_CONFIGS:
        if headline is not None and name == headline[0]:
            rows[name] = headline[1]
            continue
        a = AttnOnly(name, torch, api)
        g = capture(torch, a.launches)
        ms = event_samples(torch, lambda i: g.replay(), n_samples, warm=10)
        st = stats_us(ms, per=a.layers)
        by, fl = attention_algorithmic(a.wl)
        row = {"workload": a.text, "us_per_launch_median": st["median_us"], "us_per_launch_min": st["min_us"],
               "samples": st["samples"], "launches_per_sample": a.layers, "algorithmic_bytes": by,
               "algorithmic_flops": fl, "traffic": traffic_on_file(name),
               "plan": api.tree_verify_attention_plan(a.desc)}
        row.update(fractions(by, fl, st["median_us"], peaks))
        rows[name] = row
        del a, g
        torch.cuda.empty_cache()
    return rows


def cpu_baseline(wl_name, layers, attn_budget_s=10.0):
    """The oracle as it stands, timed on the host cores over a bounded sample of the same workload and scaled to
    one whole step.  Attention (nearly all of a step's CPU time) is timed per (sequence, layer) unit, all heads
    and rows of the sequence, until the budget is spent, and scaled by the rows x keys of the units not run;
    mask, tree tensors, gather and posterior run once over the full batch; the commit runs over one layer (all
    layers if the caches are small) and is scaled by the layer count."""
    import numpy as np
    import oracle
    wl, _ = make_host_workload(wl_name, with_cache=True)
    B = wl.B
    t0 = time.perf_counter()
    m = oracle.build_tree_mask(wl.parent, wl.n_nodes)
    tz = oracle.tensorize_tree(wl.parent, wl.n_nodes, wl.prefix_len, wl.retrieve.shape[1], wl.W)
    assert np.array_equal(tz["retrieve"], wl.retrieve)
    t_tree = time.perf_counter() - t0
    work = [int(wl.n_nodes[b]) * (int(wl.prefix_len[b]) + int(wl.n_nodes[b])) for b in range(B)]
    done_work, units, t_attn = 0, 0, 0.0
    while units < B * layers and (units == 0 or t_attn < attn_budget_s):
        b = units % B
        sl = slice(b, b + 1)
        t1 = time.perf_counter()
        oracle.tree_verify_attention(wl.q[sl], wl.k_cache if wl.paged else wl.k_cache[sl],
                                     wl.v_cache if wl.paged else wl.v_cache[sl], wl.prefix_len[sl], wl.kt[sl], wl.vt[sl],
                                     m["dense"][sl], wl.n_nodes[sl], dtype=wl.dtype,
                                     block_table=wl.block_table[sl] if wl.paged else None, want_lse=False)
        t_attn += time.perf_counter() - t1
        done_work += work[b]
        units += 1
    attn_step = t_attn * (layers * sum(work)) / done_work
    t0 = time.perf_counter()
    oracle.safe_gather_paths(wl.retrieve, wl.n_nodes, wl.T_max, 0, wl.tokens.reshape(B, wl.T_max, 1))
    p = oracle.evaluate_posterior(wl.logits, wl.tokens, wl.retrieve, wl.n_nodes)
    t_post = time.perf_counter() - t0
    cl = layers if layers * wl.k_cache.nbytes <= 2 ** 30 else 1
    kt = np.broadcast_to(wl.kt, (cl,) + wl.kt.shape).copy()
    vt = np.broadcast_to(wl.vt, (cl,) + wl.vt.shape).copy()
    kc = np.broadcast_to(wl.k_cache, (cl,) + wl.k_cache.shape).copy()
    vc = np.broadcast_to(wl.v_cache, (cl,) + wl.v_cache.shape).copy()
    t0 = time.perf_counter()
    oracle.commit_accepted_kv(kt, vt, kc, vc, wl.prefix_len, wl.capacity, wl.n_nodes, p["acc_nodes"], p["accept_len"],
                              block_table=wl.block_table)
    t_commit = (time.perf_counter() - t0) * layers / cl
    step = t_tree + attn_step + t_post + t_commit
    exact = units >= B * layers and cl == layers
    return {"value": float(wl.n_nodes.sum()) / step, "unit": "tokens/s", "cores": oracle.num_threads(),
            "kind": "oracle", "extrapolated": not exact,
            "sample": f"{wl_name}: oracle attention on {units} of {B * layers} (sequence, layer) units "
                      f"({t_attn:.1f} s, scaled by rows x keys to {attn_step:.1f} s per step); mask + tree tensors "
                      f"({t_tree:.2f} s), gather + posterior ({t_post:.2f} s) on the full batch; commit over {cl} of "
                      f"{layers} layers (scaled: {t_commit:.2f} s)",
            "seconds": t_tree + t_attn + t_post + t_commit * cl / layers, "step_seconds_estimate": step}


def main():
    a = parse_args()
    if a.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        raise SystemExit(2)
    import numpy as np
    import torch
    from paper_2603_08088_amd import api
    api.lib()   # fail loudly if the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    n_samples = max(50, a.samples)
    wl, desc_text = make_host_workload(a.workload)
    st = Step(wl, a.layers, a.sets, a.kv_split, a.attn_flags)
    tokens_per_step = int(wl.n_nodes.sum())
    if a.calib_copy_mib > 0:
        src = torch.ones(a.calib_copy_mib * 2 ** 20, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    if a.no_graph:
        runners = [(lambda s=s: st.run(s)) for s in range(st.nsets)]
    else:
        graphs = [st.capture(lambda s=s: st.run(s)) for s in range(st.nsets)]
        runners = [g.replay for g in graphs]
    for i in range(a.warmup):
        runners[i % st.nsets]()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(a.steps):
        runners[i % st.nsets]()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / a.steps

    # sanity of the step's integer results against what the generator planted
    accept = st.post_out["accept_len"].cpu().numpy().tolist()
    assert accept == [d for _, d in wl.planted], (accept, wl.planted)
    assert int(st.commit_out["status"].abs().sum().item()) == 0 and int(st.mask_out["status"].abs().sum().item()) == 0

    # median / minimum over event-timed replays: the whole step and its parts (each part its own graph)
    timing = {"whole_step": stats_us(event_samples(torch, lambda i: runners[i % st.nsets](), n_samples))}
    # dominant kernel: one tree_verify_attention launch per layer.  A sample = the step's `layers` launches back to
    # back between HIP events on the launch stream (captured as a graph of attention launches only).
    if not a.no_graph:
        att = [st.capture(lambda s=s: st.attention_layers(s)) for s in range(st.nsets)]
        att_fn = lambda i: att[i % st.nsets].replay()
        # the short parts: a sample is a graph of 20 calls (both are idempotent), so that the replay's own launch
        # cost does not drown a call of a few microseconds
        REP = 20

        def tree_calls():
            for _ in range(REP):
                api.tensorize_tree(st.parent, st.n_nodes, st.prefix_len, st.L_max, st.W, out=st.mask_out)

        def epilogue_calls():
            for _ in range(REP):
                st.epilogue(0)
        g_tree, g_epi = st.capture(tree_calls), st.capture(epilogue_calls)
        timing["tensorize_tree"] = stats_us(event_samples(torch, lambda i: g_tree.replay(), n_samples), per=REP)
        timing["verify_epilogue"] = stats_us(event_samples(torch, lambda i: g_epi.replay(), n_samples), per=REP)
    else:
        att_fn = lambda i: st.attention_layers(i % st.nsets)
    att_ms = event_samples(torch, att_fn, n_samples)
    att_stats = stats_us(att_ms, per=a.layers)
    timing["tree_verify_attention_per_launch"] = att_stats
    att_us = att_stats["mean_us"]
    by, fl = attention_algorithmic(wl)
    peaks = {} if a.no_probes else run_probes(torch)
    hbm_t, mfma_t = by / (HBM_PEAK_GBS * 1e9), fl / (MFMA_BF16_PEAK_TFLOPS * 1e12)
    if hbm_t >= mfma_t:
        roof = {"bound": "hbm", "achieved": by / (att_us * 1e-6) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s"}
    else:
        roof = {"bound": "mfma", "achieved": fl / (att_us * 1e-6) / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s"}
    roof["frac"] = roof["achieved"] / roof["peak"]
    roof["traffic"] = traffic_on_file(a.workload)
    roof["plan"] = api.tree_verify_attention_plan(st.desc)
    roof.update({"kernel": "tree_verify_attention (one layer; attn_mfma_kernel, plus attn_combine_kernel when the keys are split)",
                 "avg_launch_us": att_us, "median_launch_us": att_stats["median_us"], "min_launch_us": att_stats["min_us"],
                 "launches_timed": n_samples * a.layers, "algorithmic_bytes": by, "algorithmic_flops": fl,
                 "hbm_gbs": by / (att_us * 1e-6) / 1e9, "mfma_tflops": fl / (att_us * 1e-6) / 1e12,
                 "hbm_frac": by / (att_us * 1e-6) / 1e9 / HBM_PEAK_GBS,
                 "mfma_frac": fl / (att_us * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS})
    if peaks:
        roof.update({"measured_stream_read_gbs": peaks["stream_gbs"],
                     "measured_mfma_tflops": {"first_launch": peaks["mfma_first_launch_tflops"],
                                              "best_launch": peaks["mfma_best_launch_tflops"],
                                              "sustained": peaks["mfma_sustained_tflops"],
                                              "attention_products": peaks["mfma_attention_products_tflops"],
                                              "how": peaks["mfma_probe"] + "; attention_products = the 283 GFLOP of matrix "
                                              "instructions of the T=128 sweep cell's launch alone in a kernel, operands "
                                              "changing from product to product (median of 100 launches)"},
                     "hbm_frac_of_measured": roof["hbm_gbs"] / peaks["stream_gbs"],
                     "mfma_frac_of_measured": roof["mfma_tflops"] / peaks["mfma_sustained_tflops"]})

    configs = None
    if not a.no_configs and not a.no_graph:
        head_row = {"workload": desc_text, "us_per_launch_median": att_stats["median_us"],
                    "us_per_launch_min": att_stats["min_us"], "samples": att_stats["samples"],
                    "launches_per_sample": a.layers, "algorithmic_bytes": by, "algorithmic_flops": fl,
                    "traffic": roof["traffic"], "plan": api.tree_verify_attention_plan(st.desc)}
        head_row.update(fractions(by, fl, att_stats["median_us"], peaks))
        configs = configs_table(torch, api, n_samples, peaks,
                                headline=(a.workload, head_row) if a.layers == 32 and not a.kv_split and not a.attn_flags else None)
    # beside the step (not part of it: the step takes logits as input): the teacher head fused with the greedy
    # choice on the step's node rows, a 7B-class head (D = 4096, V = the workload's vocabulary), weights packed once
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    head = None
    if not a.no_lm_head:
        Dm, V = 4096, wl.V
        hid = torch.randn((wl.B, wl.T_max, Dm), device="cuda:0").to(torch.bfloat16)
        nsets = max(1, -(-640 * 2 ** 20 // (2 * V * Dm)))     # rotate so that the weights stream from HBM
        packed = []
        for _ in range(nsets):
            wt = (torch.randn((V, Dm), device="cuda:0") / 64).to(torch.bfloat16)
            packed.append(api.pack_lm_head(wt))
            del wt
        hws = torch.empty((max(256, int(api.lib().etv_lm_head_argmax_workspace_bytes(wl.B, wl.T_max, V))),),
                          dtype=torch.uint8, device="cuda:0")
        hout = dict(argmax=torch.empty((wl.B, wl.T_max), dtype=torch.int32, device="cuda:0"),
                    maxval=torch.empty((wl.B, wl.T_max), dtype=torch.float32, device="cuda:0"))

        def head_call(i):
            api.lm_head_argmax(hid, packed[i % nsets], st.n_nodes, V=V, workspace=hws, out=hout)
        for i in range(3):
            head_call(i)
        torch.cuda.synchronize()
        e0.record()
        for i in range(20):
            head_call(i)
        e1.record()
        torch.cuda.synchronize()
        head_us = e0.elapsed_time(e1) * 1e3 / 20
        e0.record()
        for i in range(20):   # the weight pass alone: the fused epilogue can finish the choice per node itself
            api.lm_head_argmax(hid, packed[i % nsets], st.n_nodes, V=V, workspace=hws, finish=False)
        e1.record()
        torch.cuda.synchronize()
        pass_us = e0.elapsed_time(e1) * 1e3 / 20
        head = {"kernel": "lm_head_argmax (head GEMM + argmax, logits never written; + finishing launch)",
                "rows": int(wl.B * wl.T_max), "D": Dm, "V": V, "us_per_call": head_us,
                "us_weight_pass_only": pass_us, "weight_bytes": 2 * V * Dm,
                "hbm_gbs": 2 * V * Dm / (head_us * 1e-6) / 1e9,
                "hbm_gbs_weight_pass_only": 2 * V * Dm / (pass_us * 1e-6) / 1e9,
                "frac_of_peak": 2 * V * Dm / (head_us * 1e-6) / 1e9 / HBM_PEAK_GBS,
                "frac_of_peak_weight_pass_only": 2 * V * Dm / (pass_us * 1e-6) / 1e9 / HBM_PEAK_GBS,
                "flops": 2.0 * tokens_per_step * V * Dm,
                "mfma_tflops": 2.0 * tokens_per_step * V * Dm / (head_us * 1e-6) / 1e12,
                "mfma_frac": 2.0 * tokens_per_step * V * Dm / (head_us * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS}
        del packed


    # beside the step as well: the branch-cache calls on a paged pool of 7B-class shape (8 KV heads, d = 128, bf16,
    # all layers): copy-on-write replication into N branches, the commit by path indices with the prefix shared
    # (the common case) and as the general full reorder (every row moved: an HBM copy)
    branch = None
    if not a.no_branch_cache:
        Bb, Nb, Pb, Tb, Hb, db, bsz, Lb = 8, 4, 2040, 60, 8, 128, 16, a.layers
        per_seq = -(-(Pb + Tb) // bsz)
        nblk = Bb * per_seq * 2 + Bb * Nb * 8 + 64
        gen = torch.Generator(device="cuda:0").manual_seed(7)
        pool_k = torch.empty((Lb, nblk, Hb, bsz, db), dtype=torch.bfloat16, device="cuda:0").normal_(generator=gen)
        pool_v = torch.empty_like(pool_k).normal_(generator=gen)
        ids = torch.randperm(nblk, generator=torch.Generator().manual_seed(7)).to(torch.int32)
        table = ids[: Bb * per_seq].reshape(Bb, per_seq).contiguous().to("cuda:0")
        free = ids[Bb * per_seq:].contiguous().to("cuda:0")
        plen = torch.full((Bb,), Pb, dtype=torch.int32, device="cuda:0")
        tlen = torch.full((Bb,), Tb, dtype=torch.int32, device="cuda:0")

        def timed(fn, n=20):
            for _ in range(3):
                fn()
            torch.cuda.synchronize()
            e0.record()
            for _ in range(n):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) * 1e3 / n
        rep = api.replicate_branches(pool_k, pool_v, table, plen, tlen, Nb, free)
        assert int(rep["status"].abs().sum().item()) == 0
        taken = int(rep["n_taken"].item())
        # each call is captured in a HIP graph like the step, so the figures are device time, not the binding's
        g_rep = st.capture(lambda: api.replicate_branches(pool_k, pool_v, table, plen, tlen, Nb, free))
        repl_us = timed(g_rep.replay)
        src_t = rep["branch_table"][:, 1].contiguous()
        dst_t = torch.full_like(src_t, -1)
        dst_t[:, :per_seq] = free[taken: taken + Bb * per_seq].reshape(Bb, per_seq)
        Ln = Pb + 6                                    # the root and five accepted draft tokens
        pidx = torch.arange(Ln, dtype=torch.int32).repeat(Bb, 1)
        pidx[:, Pb:] = Pb + torch.tensor([0, 2, 7, 19, 33, 51], dtype=torch.int32)
        pidx = pidx.to("cuda:0")
        slen = torch.full((Bb,), Pb + Tb, dtype=torch.int32, device="cuda:0")
        nlen = torch.full((Bb,), Ln, dtype=torch.int32, device="cuda:0")
        keep_t = dst_t.clone()

        def path_commit(fast):
            dst_t.copy_(keep_t)
            return api.commit_path_indices(pool_k, pool_v, pool_k, pool_v, pidx, slen, nlen, src_table=src_t,
                                           dst_table=dst_t, fast=fast)
        r = path_commit(True)
        assert int(r["status"].abs().sum().item()) == 0 and int(r["kept_len"][0].item()) == Pb // bsz * bsz
        g_tab, g_fast = st.capture(lambda: dst_t.copy_(keep_t)), st.capture(lambda: path_commit(True))
        g_full = st.capture(lambda: path_commit(False))
        table_us = timed(g_tab.replay)                 # restoring the destination table is not part of the call
        fast_us = timed(g_fast.replay) - table_us
        full_us = timed(g_full.replay, n=5) - table_us
        moved = 2 * 2 * Ln * Hb * db * 2 * Lb * Bb       # read + write, K and V, every row, every layer, every sequence
        branch = {"shape": f"B={Bb} N={Nb} P={Pb} T={Tb} Hkv={Hb} d={db} bf16 block={bsz} layers={Lb}",
                  "replicate_us": repl_us, "deep_copy_bytes_avoided": 2 * Pb * Hb * db * 2 * Lb * Bb * Nb,
                  "commit_path_indices_fast_us": fast_us, "commit_path_indices_full_reorder_us": full_us,
                  "full_reorder_bytes": moved, "full_reorder_hbm_gbs": moved / (full_us * 1e-6) / 1e9,
                  "full_reorder_frac_of_peak": moved / (full_us * 1e-6) / 1e9 / HBM_PEAK_GBS}
        del pool_k, pool_v

    cpu = None if a.skip_cpu else cpu_baseline(a.workload, a.layers)
    line = {
        "metric": "tree-verify tokens/s (batch x tree nodes)", "value": tokens_per_step / (ms_per_step * 1e-3),
        "unit": "tokens/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": f"{a.workload}: {desc_text}", "layers": a.layers, "tokens_per_step": tokens_per_step,
                   "launch": "eager" if a.no_graph else "hip-graph replay", "cache_sets": st.nsets,
                   "cache_bytes": st.cache_bytes, "kv_split": a.kv_split},
        "roofline": roof, "cpu_baseline": cpu, "timing": timing, "configs": configs, "lm_head_argmax": head,
        "branch_cache": branch,
    }
    # The full report (every figure, the plans, the sample descriptions) goes to the file named by --report ("-":
    # stderr); stdout carries ONE compact JSON line with the same keys: numbers rounded to four significant digits, the
    # per-configuration table as rows of [median us, min us, HBM fraction, MFMA fraction, counter traffic /
    # algorithmic bytes], so that the line stays a few KB for whatever reads the tail of the output.
    if a.report == "-":
        print("bench report: " + json.dumps(line), file=sys.stderr, flush=True)
    elif a.report:
        with open(a.report, "w") as f:
            json.dump(line, f, indent=1)
    print(json.dumps(compact(line)), flush=True)


def compact(line):
    def r4(x):
        if isinstance(x, float):
            return float(f"{x:.4g}")
        if isinstance(x, dict):
            return {k: r4(v) for k, v in x.items()}
        if isinstance(x, list):
            return [r4(v) for v in x]
        return x
    out = {k: line[k] for k in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better",
                                "scaling", "vs_baseline", "dtype", "data")}
    out["config"] = {k: line["config"][k] for k in ("workload", "layers", "tokens_per_step", "launch")}
    roof = dict(line["roofline"])
    roof.pop("plan", None)
    m = roof.get("measured_mfma_tflops")
    if m:
        roof["measured_mfma_tflops"] = {k: m[k] for k in ("first_launch", "sustained", "attention_products")}
    roof["kernel"] = "tree_verify_attention (attn_mfma_kernel)"
    out["roofline"] = r4(roof)
    cpu = line["cpu_baseline"]
    if cpu:
        cpu = dict(cpu)
        cpu["sample"] = cpu["sample"][:160]
        cpu.pop("seconds", None)
    out["cpu_baseline"] = r4(cpu)
    out["timing_us_median_min"] = {k: [r4(v["median_us"]), r4(v["min_us"])] for k, v in line["timing"].items()}
    out["timing_samples"] = min(v["samples"] for v in line["timing"].values())
    if line["configs"]:
        out["configs_columns"] = ["us_per_launch_median", "us_per_launch_min", "hbm_frac", "mfma_frac",
                                  "traffic_over_algorithmic_bytes"]
        out["configs"] = {k: [r4(v["us_per_launch_median"]), r4(v["us_per_launch_min"]), r4(v["hbm_frac"]),
                              r4(v["mfma_frac"]),
                              r4(v["traffic"] / v["algorithmic_bytes"]) if v["traffic"] else None]
                          for k, v in line["configs"].items()}
    h = line["lm_head_argmax"]
    if h:
        out["lm_head_argmax"] = r4({k: h[k] for k in ("rows", "us_per_call", "mfma_tflops", "hbm_gbs")})
    b = line["branch_cache"]
    if b:
        out["branch_cache"] = r4({k: b[k] for k in ("replicate_us", "commit_path_indices_fast_us",
                                                    "commit_path_indices_full_reorder_us", "full_reorder_hbm_gbs")})
    return out


if __name__ == "__main__":
    main()
