#!/usr/bin/env python3
"""Benchmark of the tree-verification hot path on one MI355X.

A "step" is one verification step of speculative decoding at the LLaMA3-8B
shape (workload c3_llama3_8b): the tree-masked attention of all `--layers`
transformer layers (32 distinct bf16 KV caches, 4096-token prefix, 60-node
two-expert draft tree, 32 query / 8 KV heads, head_dim 128) followed by one
acceptance walk over [61, 128256] fp32 logits (temperature-1 speculative
sampling).  Inputs are synthetic, seeded, and resident in HBM before the timed
region.  The KV ring (layers x 16.8 MB = 537 MB at 32 layers) is larger than
the 256 MB Infinity Cache, so every attention call streams its KV from HBM.

Prints one JSON line.  `value` is the attention's algorithmic bytes per second
(KV prefix + tree K/V + Q + O, 18 006 016 B per call) over the time the step
spends in attention calls; `ms_per_step` covers the whole step.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0

# HBM bytes per launch of the attention kernel (tva_bf16_kernel; for c5 without its merge kernel) from
# rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs (KiB per dispatch), each scaled by the same counter's reading
# for a 256 MiB device copy (factors 2.00 and 1.00); source: profiles/<workload>_attention_and_acceptance.md.
# {workload: bytes}; None for workloads that were not measured.
MEASURED_TRAFFIC = {"c2_vicuna7b": 26704104, "c3_llama3_8b": 34393582, "c4_llama2_13b": 191863442,
                    "c5_llama2_70b": 714200829, "c6_chain_sps": 269956059,
                    "c7_static_tree": 77957017}


def attn_bytes(cfg) -> int:
    es = 2 if cfg.dtype == "bf16" else 4
    L, T, Hq, Hkv, D = cfg.prefix_len, cfg.n_tree, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    return cfg.batch * (2 * L * Hkv * D * es + 2 * T * Hkv * D * es + 2 * T * Hq * D * es)


def device_state():
    """Clock and power state as rocm-smi reports it after the run (None if the tool is missing)."""
    import subprocess
    # (under a profiler's preloaded library every child process has the GPU initialised before it starts, and the
    # tool is a script that re-executes an interpreter: not started from such a process)
    if "rocprof" in os.environ.get("LD_PRELOAD", "").lower() or any(k.startswith(("ROCPROF", "ROCP_")) for k in os.environ):
        return None
    try:
        r = subprocess.run(["rocm-smi", "--showclocks", "--showpower", "--json"], capture_output=True, text=True, timeout=20)
        d = json.loads(r.stdout)
        card = d.get("card0", next(iter(d.values())))
        keep = {k: v for k, v in card.items() if any(t in k.lower() for t in ("sclk", "mclk", "power"))}
        return keep or None
    except Exception:
        return None


def _one_blas_thread():
    """Pool initializer: a worker computes its unit on one thread (the pool is the parallelism)."""
    try:
        from threadpoolctl import threadpool_limits
        threadpool_limits(limits=1)
    except Exception:  # pragma: no cover
        pass


def _oracle_unit(job):
    """One (sequence, KV head) unit of the attention oracle (worker of the all-cores leg)."""
    from oracle import tree_verify_attention as o_attn
    x, par_b, L = job
    return o_attn(**x, parent=par_b, prefix_len=[L]).shape


def _unit_jobs(cfg, x, par):
    G = cfg.n_q_heads // cfg.n_kv_heads
    jobs = []
    for b in range(cfg.batch):
        for h in range(cfg.n_kv_heads):
            jobs.append(({"q": x["q"][b:b + 1, :, h * G:(h + 1) * G], "k_cache": x["k_cache"][b:b + 1, :, h:h + 1],
                          "v_cache": x["v_cache"][b:b + 1, :, h:h + 1], "k_tree": x["k_tree"][b:b + 1, :, h:h + 1],
                          "v_tree": x["v_tree"][b:b + 1, :, h:h + 1]}, par[b:b + 1], cfg.prefix_len))
    return jobs


def cpu_baseline(cfg, par, x0, acc, budget_s=8.0):
    """The oracle as it stands on a bounded sample of the same workload, in the metric's unit (algorithmic
    attention bytes per second): (a) one thread: the attention of whole layers (all heads) until about
    `budget_s` seconds are spent, and one acceptance walk; (b) all host cores this box gives a one-GPU job
    (at most 16 processes), one (sequence, KV head) unit of a layer per task, for about as long.  The
    all-cores figure is the reported `value`; the one-thread figure sits beside it."""
    import multiprocessing as mp
    from oracle import accept_path as o_accept, tree_verify_attention as o_attn
    from workloads import attention_inputs
    try:
        from threadpoolctl import threadpool_limits
    except Exception:  # pragma: no cover
        threadpool_limits = None

    jobs = _unit_jobs(cfg, x0, par)

    def run():
        # (sequence, KV head) units of one layer after the other, further layers while the budget lasts
        t_attn, n_units, layer = 0.0, 0, 0
        while t_attn < budget_s and layer < 32:
            js = jobs if layer == 0 else _unit_jobs(cfg, attention_inputs(cfg, layer=layer), par)   # generation is not timed
            for x, par_b, L in js:
                t0 = time.perf_counter()
                o_attn(**x, parent=par_b, prefix_len=[L])
                t_attn += time.perf_counter() - t0
                n_units += 1
                if t_attn >= budget_s:
                    break
            layer += 1
        t0 = time.perf_counter()
        walks = []
        for b in range(cfg.batch):
            walks.append(o_accept(acc["tokens"][b], par[b], acc["logits"][b], cfg.mode,
                                  None if acc["draft_probs"] is None else acc["draft_probs"][b],
                                  None if acc["uniforms"] is None else acc["uniforms"][b]))
        return t_attn, n_units, time.perf_counter() - t0, walks

    if threadpool_limits is not None:
        with threadpool_limits(limits=1):
            t_attn, n_done, t_acc, walks = run()
    else:
        t_attn, n_done, t_acc, walks = run()
    layers_done = n_done / len(jobs)
    one = {"value": round(attn_bytes(cfg) * layers_done / t_attn / 1e9, 4), "cores": 1,
           "attention_us_per_call": round(t_attn / layers_done * 1e6, 1),
           "sample": f"{n_done} (sequence, KV head) units = {layers_done:.2f} layers' attention ({t_attn:.1f} s) + one acceptance "
                     f"walk ({t_acc * 1e3:.1f} ms)"}

    # (b) all cores: tasks are independent (sequence, KV head) units; each worker keeps BLAS to one thread
    cores = max(1, min(os.cpu_count() or 1, 16))
    t_par, n_units = 0.0, 0
    if cores > 1:
        ctx = mp.get_context("fork")
        with ctx.Pool(cores, initializer=_one_blas_thread) as pool:
            pool.map(_oracle_unit, jobs[:cores])  # start-up of the workers is not timed
            while t_par < budget_s:
                t0 = time.perf_counter()
                pool.map(_oracle_unit, jobs, chunksize=1)
                t_par += time.perf_counter() - t0
                n_units += len(jobs)
    if n_units:
        per_layer = t_par / (n_units / len(jobs))
        value, used, us_call = attn_bytes(cfg) / per_layer / 1e9, cores, per_layer * 1e6
        sample = (f"fp64 NumPy oracle on {cores} processes, one (sequence, KV head) unit per task: {n_units // len(jobs)} "
                  f"full layer(s) in {t_par:.1f} s; beside it one thread: {one['sample']}")
    else:
        value, used, us_call, sample = one["value"], 1, one["attention_us_per_call"], "fp64 NumPy oracle, one thread: " + one["sample"]
    # what the realised sampling walk touches: the logits rows of the nodes it stands on and, per rejected
    # sibling, that sibling's draft row (an accepted child costs two scalars)
    touched = None
    if cfg.mode == "sample":
        rows = sum(w.accept_len + 1 for w in walks)
        rejects = sum(sum(1 for d in w.decisions if d[0] == "reject") for w in walks)
        touched = (rows + rejects) * cfg.vocab * 4
    return {
        "value": round(value, 4),
        "unit": "GB/s",
        "cores": used,
        "kind": "oracle",
        "sample": sample,
        "attention_us_per_call": round(us_call, 1),
        "single_thread": one,
        "host_cpu_count": os.cpu_count(),
        "accept_nodes_per_s": round(cfg.batch * cfg.n_tree / t_acc, 1),
        "accept_walk": {"accept_len": [w.accept_len for w in walks], "bytes_touched_by_the_walk": touched},
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--layers", type=int, default=0, help="attention calls (distinct KV buffers) per step; "
                    "default: the model's depth (32; 40 for c4; 2 x 537 MB for c5)")
    ap.add_argument("--workload", default="c3_llama3_8b")
    ap.add_argument("--paged", type=int, default=0, metavar="PAGE_SIZE",
                    help="keep the KV caches in page pools of this page size (a multiple of 32) with a shuffled "
                         "block table and time jk_tree_verify_attention_paged instead")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-draft-heads", action="store_true", help="skip the jk_draft_heads timing (extra field)")
    ap.add_argument("--draft-rows", type=int, default=0, help="hidden states per jk_draft_heads call "
                    "(default: 10 per sequence of the workload)")
    ap.add_argument("--kv-layout", choices=("token", "head"), default="token",
                    help="storage order of the K/V caches: [B, L, Hkv, D] (token-major, the default) or "
                    "[B, Hkv, L, D] (head-major: each KV head's stream contiguous), passed through the strides")
    ap.add_argument("--no-graph", action="store_true", help="issue every library call from Python instead of "
                    "replaying the step's two HIP graphs")
    ap.add_argument("--copy-calibration", type=int, default=0,
                    help="also run this many 256 MiB device copies (reference kernel for --pmc runs)")
    ap.add_argument("--no-extras", action="store_true", help="skip the side measurements (cold / warm-cache launches, "
                    "repetitions, deep walk, probes, commit, draft side): only the timed steps")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (--gpus 1); there is no multi-GPU path to time")

    import numpy as np

    from workloads import CONFIGS, accept_inputs, attention_inputs, tree_for_config

    cfg = CONFIGS[args.workload]
    if args.layers <= 0:
        args.layers = {"c4_llama2_13b": 40, "c5_llama2_70b": 2, "c1_tiny": 32, "c6_chain_sps": 4, "c7_static_tree": 16}.get(cfg.name, 32)
    par = tree_for_config(cfg)
    acc = accept_inputs(cfg, par)
    # The oracle's timing comes first, before this process touches the GPU (its all-cores leg forks workers).
    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(cfg, par, attention_inputs(cfg, layer=0), acc)

    import torch

    import paper_2502_06282_amd as jk

    jk.lib()  # fail loudly if the HIP library is missing
    dev = torch.device("cuda:0")
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    parent = torch.from_numpy(par).to(dev)
    plen = torch.full((cfg.batch,), cfg.prefix_len, dtype=torch.int32, device=dev)

    layers = []
    for l in range(args.layers):
        x = attention_inputs(cfg, layer=l)
        layers.append({k: torch.from_numpy(v).to(dev).to(tdt) for k, v in x.items()})
        if args.kv_layout == "head":
            for name in ("k_cache", "v_cache"):
                layers[-1][name] = layers[-1][name].permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    mode = jk.JK_GREEDY if cfg.mode == "greedy" else jk.JK_SAMPLE
    tokens = torch.from_numpy(acc["tokens"]).to(dev)
    logits = torch.from_numpy(acc["logits"]).to(dev)
    draft = None if acc["draft_probs"] is None else torch.from_numpy(acc["draft_probs"]).to(dev)
    unif = None if acc["uniforms"] is None else torch.from_numpy(acc["uniforms"]).to(dev)

    out = torch.empty_like(layers[0]["q"])
    ws_attn = torch.empty(jk.tree_verify_attention_workspace(layers[0]["q"], layers[0]["k_cache"],
                                                             layers[0]["k_tree"], cfg.prefix_len),
                          dtype=torch.uint8, device=dev)
    jk.workspace_init(ws_attn)
    ws_acc = torch.empty(jk.accept_path_workspace(cfg.batch, cfg.n_tree, cfg.vocab, mode), dtype=torch.uint8,
                         device=dev)
    jk.workspace_init(ws_acc)

    o_path = torch.empty((cfg.batch, cfg.depth), dtype=torch.int32, device=dev)
    o_len = torch.empty((cfg.batch,), dtype=torch.int32, device=dev)
    o_bonus = torch.empty((cfg.batch,), dtype=torch.int32, device=dev)
    if args.paged:
        # the same cache contents, page by page at shuffled places of a pool (one table for all layers)
        ps = args.paged
        nb = (cfg.prefix_len + ps - 1) // ps
        n_pages = cfg.batch * nb + 3
        perm = torch.randperm(n_pages, generator=torch.Generator().manual_seed(0))[: cfg.batch * nb]
        table = perm.to(torch.int32).reshape(cfg.batch, nb).to(dev)
        for lyr in layers:
            for name in ("k_cache", "v_cache"):
                c = lyr[name]
                pad = nb * ps - cfg.prefix_len
                if pad:
                    c = torch.cat([c, torch.zeros((cfg.batch, pad) + tuple(c.shape[2:]), dtype=c.dtype, device=dev)], 1)
                pool = torch.zeros((n_pages, ps) + tuple(c.shape[2:]), dtype=c.dtype, device=dev)
                pool[table.reshape(-1).long()] = c.reshape(cfg.batch * nb, ps, *c.shape[2:])
                lyr[name + "_pool"] = pool
        attn_calls = [jk.prepare_tree_verify_attention_paged(lyr["q"], lyr["k_cache_pool"], lyr["v_cache_pool"], table,
                                                             lyr["k_tree"], lyr["v_tree"], parent, plen, out, ws_attn,
                                                             max_prefix_len=cfg.prefix_len) for lyr in layers]
    else:
        attn_calls = [jk.prepare_tree_verify_attention(lyr["q"], lyr["k_cache"], lyr["v_cache"], lyr["k_tree"],
                                                       lyr["v_tree"], parent, plen, out, ws_attn,
                                                       max_prefix_len=cfg.prefix_len) for lyr in layers]
    acc_call = jk.prepare_accept_path(tokens, parent, logits, mode, 1.0, draft, unif, o_path, o_len, o_bonus, ws_acc)
    res = (o_path, o_len, o_bonus)

    def attention_eager():
        for c in attn_calls:
            c.launch()

    attention_pass, accept_pass = attention_eager, acc_call.launch
    if not args.no_graph:
        # one HIP graph per phase: the step's launches replay without per-call host work,
        # as a serving loop would issue them
        attention_eager(); acc_call.launch()
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        g_attn, g_acc = torch.cuda.CUDAGraph(), torch.cuda.CUDAGraph()
        with torch.cuda.graph(g_attn, stream=side):
            attention_eager()
        with torch.cuda.graph(g_acc, stream=side):
            acc_call.launch()
        attention_pass, accept_pass = g_attn.replay, g_acc.replay

    for _ in range(args.warmup):
        attention_pass()
        accept_pass()
    torch.cuda.synchronize()

    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for s in range(args.steps):
        ev[s][0].record()
        attention_pass()
        ev[s][1].record()
        accept_pass()
        ev[s][2].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    t_attn_ms = sum(e[0].elapsed_time(e[1]) for e in ev) / args.steps
    t_acc_ms = sum(e[1].elapsed_time(e[2]) for e in ev) / args.steps
    ms_per_step = wall * 1e3 / args.steps
    per_call_us = t_attn_ms * 1e3 / args.layers
    bytes_call = attn_bytes(cfg)
    gbps = bytes_call / (per_call_us * 1e-6) / 1e9
    flops_call = 4.0 * cfg.batch * cfg.n_tree * cfg.n_q_heads * (cfg.prefix_len + cfg.n_tree) * cfg.head_dim
    tflops = flops_call / (per_call_us * 1e-6) / 1e12
    plan = jk.tree_verify_attention_plan(layers[0]["q"], layers[0]["k_cache"], layers[0]["k_tree"], cfg.prefix_len)

    def timed_us(fn, reps, per):
        """[us per unit] of `reps` runs of fn (HIP events on the current stream around each run)."""
        out_us = []
        for _ in range(reps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(); fn(); b.record()
            torch.cuda.synchronize()
            out_us.append(a.elapsed_time(b) * 1e3 / per)
        return out_us

    timing = None
    if not args.no_extras and not args.no_graph:
        # M-TIME: five repetitions of the attention phase of a step (steady state: every call streams its K/V
        # from HBM, the ring of layers is larger than the Infinity Cache); one call alone, after everything
        # else has drained and its buffers were last touched a ring ago ("cold": includes what a lone launch
        # costs); the same call over and over (K/V served by the Infinity Cache: NOT an HBM figure)
        reps = sorted(timed_us(attention_pass, 5, args.layers))
        torch.cuda.synchronize()
        cold = timed_us(attn_calls[len(attn_calls) // 2].launch, 1, 1)[0]
        warm_call = attn_calls[0]
        def warm_pass():
            for _ in range(16):
                warm_call.launch()
        warm_pass(); torch.cuda.synchronize()
        g_warm = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g_warm, stream=torch.cuda.Stream()):
            warm_pass()
        g_warm.replay(); torch.cuda.synchronize()
        warm = sorted(timed_us(g_warm.replay, 5, 16))
        timing = {"steady_us_per_call_median_of_5": round(reps[2], 3), "steady_us_per_call_min_of_5": round(reps[0], 3),
                  "cold_single_launch_us": round(cold, 2),
                  "warm_cache_us_per_call_median_of_5": round(warm[2], 3),
                  "note": "steady: graph replay over the ring of layers (HBM); cold: one eager call, device idle before "
                          "it; warm_cache: the same layer's call 16 times per replay, its K/V resident in the "
                          "Infinity Cache - not an HBM figure"}

    probe = commit = deep = acc_b2b = None
    if not args.no_extras:
        # ceiling for one layer's K/V on this machine: a kernel that only streams as many bytes as one
        # layer's K and V prefix (16.8 MB), from its own ring of buffers larger than the Infinity Cache
        sink = torch.zeros(4, dtype=torch.int32, device=dev)
        probe_bytes = 2 * layers[0]["k_cache"].numel() * layers[0]["k_cache"].element_size()
        probe_ring = [torch.full((probe_bytes,), 1, dtype=torch.uint8, device=dev) for _ in range(args.layers)]
        def stream_pass():
            for buf in probe_ring:
                jk.stream_read_probe(buf, sink)
        stream_pass()
        torch.cuda.synchronize()
        g_probe = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g_probe, stream=torch.cuda.Stream()):
            stream_pass()
        g_probe.replay()
        torch.cuda.synchronize()
        es0, es1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        es0.record()
        for _ in range(5):
            g_probe.replay()
        es1.record()
        torch.cuda.synchronize()
        probe_us = es0.elapsed_time(es1) * 1e3 / (5 * args.layers)
        # the same probe on 16 bytes: what a launch costs on its own in this chain of dependent launches
        tiny = torch.zeros(16, dtype=torch.uint8, device=dev)
        def floor_pass():
            for _ in range(args.layers):
                jk.stream_read_probe(tiny, sink)
        floor_pass(); torch.cuda.synchronize()
        g_floor = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g_floor, stream=torch.cuda.Stream()):
            floor_pass()
        g_floor.replay(); torch.cuda.synchronize()
        es0.record()
        for _ in range(5):
            g_floor.replay()
        es1.record()
        torch.cuda.synchronize()
        floor_us = es0.elapsed_time(es1) * 1e3 / (5 * args.layers)
        # the step after the path (not part of the timed step): commit of a full-depth accepted path to
        # every layer's cache in one call, rows landing in the last `depth` rows of the caches, length not advanced
        chain = []
        for i in range(cfg.n_tree):
            c, a = [], i
            while a >= 0:
                c.append(a)
                a = int(par[0, a])
            if len(c) > len(chain):
                chain = c[::-1]
        chain = (chain + [-1] * cfg.depth)[:cfg.depth]
        n_commit = sum(1 for v in chain if v >= 0)
        c_path = torch.tensor([chain] * cfg.batch, dtype=torch.int32, device=dev)
        c_len = torch.full((cfg.batch,), n_commit, dtype=torch.int32, device=dev)
        c_plen = torch.full((cfg.batch,), cfg.prefix_len - n_commit, dtype=torch.int32, device=dev)
        commit_call = jk.prepare_commit_path_layers([lyr["k_tree"] for lyr in layers], [lyr["v_tree"] for lyr in layers],
                                                    [lyr["k_cache"] for lyr in layers], [lyr["v_cache"] for lyr in layers],
                                                    c_path, c_len, c_plen, advance=False)
        def commit_pass():  # 16 calls per graph replay, so that the replay's own cost does not hide the call's
            for _ in range(16):
                commit_call.launch()
        commit_pass()
        torch.cuda.synchronize()
        g_commit = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g_commit, stream=torch.cuda.Stream()):
            commit_pass()
        g_commit.replay()
        torch.cuda.synchronize()
        ec0, ec1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ec0.record()
        for _ in range(5):
            g_commit.replay()
        ec1.record()
        torch.cuda.synchronize()
        commit_us = ec0.elapsed_time(ec1) * 1e3 / (5 * 16)
        commit_bytes = args.layers * 4 * cfg.batch * n_commit * cfg.n_kv_heads * cfg.head_dim * layers[0]["k_cache"].element_size()
        probe = {"bytes_per_launch": probe_bytes, "us_per_launch": round(probe_us, 3),
                 "GBps": round(probe_bytes / (probe_us * 1e-6) / 1e9, 1), "empty_launch_us": round(floor_us, 3),
                 "note": "pure 128-bit read kernel, one launch per buffer (one layer's K/V bytes) of a ring of as many "
                         "buffers as layers, HIP-graph replay; empty_launch_us: the same kernel on 16 bytes, i.e. the "
                         "cost of a launch in a chain of dependent launches"}
        commit = {"us_per_call": round(commit_us, 3), "rows_per_sequence": n_commit, "bytes_per_call": commit_bytes,
                  "layers": args.layers,
                  "note": "one jk_commit_path_layers call for all layers after the step (not in ms_per_step)"}
        # the acceptance call eight times in one graph: what a call costs when it sits among other launches
        # of a round's graph (the step's figure is one call per graph replay and carries the replay's own
        # launch latency)
        def acc8():
            for _ in range(8):
                acc_call.launch()
        acc8(); torch.cuda.synchronize()
        g_acc8 = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g_acc8, stream=torch.cuda.Stream()):
            acc8()
        g_acc8.replay(); torch.cuda.synchronize()
        acc_b2b = sorted(timed_us(g_acc8.replay, 5, 8))[2]
        if mode == jk.JK_SAMPLE:
            # a walk that goes deep: draft distributions close to the target's (0.97 softmax(parent row) + 0.03 q)
            # and every first child carrying its parent row's likeliest token; the timed step above uses the
            # workload's own Dirichlet(0.1) drafts, whose walk ends after a handful of rejections at depth 1
            lg = acc["logits"].astype(np.float64)
            q2, tok2 = acc["draft_probs"].copy(), acc["tokens"].copy()
            for b_ in range(cfg.batch):
                for k in range(cfg.n_tree):
                    row = lg[b_, par[b_, k] + 1]
                    e = np.exp(row - row.max())
                    q2[b_, k] = (0.97 * e / e.sum() + 0.03 * q2[b_, k]).astype(np.float32)
                    if k == int(np.nonzero(par[b_] == par[b_, k])[0][0]):
                        tok2[b_, k] = int(np.argmax(row))
            d_tok, d_q = torch.from_numpy(tok2).to(dev), torch.from_numpy(q2).to(dev)
            deep_call = jk.prepare_accept_path(d_tok, parent, logits, mode, 1.0, d_q, unif, o_path, o_len, o_bonus, ws_acc)
            deep_call.launch(); torch.cuda.synchronize()
            deep_len = [int(v) for v in o_len.cpu().tolist()]
            g_deep = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g_deep, stream=torch.cuda.Stream()):
                deep_call.launch()
            g_deep.replay(); torch.cuda.synchronize()
            deep_us = sorted(timed_us(g_deep.replay, 5, 1))
            deep = {"us_per_call_median_of_5": round(deep_us[2], 2), "accept_len": deep_len,
                    "note": "the same logits with draft distributions close to the target's: a walk that descends"}
            acc_call.launch(); torch.cuda.synchronize()   # (outputs of the workload's own walk again)
            del d_q
    # the step in front of the path (not part of the timed step): both draft heads over the shared
    # output embedding for the nodes one draft step expands (10 per sequence), random weights
    draft = None
    if not args.no_draft_heads and not args.no_extras:
        dh_rows = min(128, args.draft_rows if args.draft_rows > 0 else 10 * cfg.batch)
        d_model = cfg.n_q_heads * cfg.head_dim
        gen = torch.Generator(device=dev).manual_seed(cfg.seed)
        dh_f = torch.randn((dh_rows, 2, d_model), device=dev, generator=gen).to(torch.bfloat16)
        dh_s = torch.rand((dh_rows, 2), device=dev, generator=gen) * 0.5
        dh_w = (torch.randn((cfg.vocab, d_model), device=dev, generator=gen) * (5.0 / d_model ** 0.5)).to(torch.bfloat16)
        dh_lg = torch.empty((dh_rows, 2, cfg.vocab), device=dev)
        dh_q = torch.empty((dh_rows, 2, cfg.vocab), device=dev)
        dh_tk = torch.empty((dh_rows, 2, 10), dtype=torch.int32, device=dev)
        dh_tp = torch.empty((dh_rows, 2, 10), device=dev)
        dh_ws = torch.empty(jk.draft_heads_workspace(dh_rows, d_model, cfg.vocab), dtype=torch.uint8, device=dev)
        dh_call = jk.prepare_draft_heads(dh_f, dh_s, dh_w, jk.JK_HEADS_DECOUPLED, 1.0, 10, 0.0, 0.0, dh_lg, dh_q,
                                         dh_tk, dh_tp, dh_ws)
        def draft_pass():
            for _ in range(4):
                dh_call.launch()
        draft_pass()
        torch.cuda.synchronize()
        g_draft = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g_draft, stream=torch.cuda.Stream()):
            draft_pass()
        g_draft.replay()
        torch.cuda.synchronize()
        ed0, ed1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ed0.record()
        for _ in range(5):
            g_draft.replay()
        ed1.record()
        torch.cuda.synchronize()
        dh_us = ed0.elapsed_time(ed1) * 1e3 / 20
        w_bytes = cfg.vocab * d_model * 2
        draft = {"us_per_call": round(dh_us, 1), "rows": dh_rows, "d_model": d_model, "vocab": cfg.vocab, "top_k": 10,
                 "weight_stream_GBps": round(w_bytes / (dh_us * 1e-6) / 1e9, 1),
                 "TFLOPs": round(4.0 * dh_rows * d_model * cfg.vocab / (dh_us * 1e-6) / 1e12, 1),
                 "note": "one jk_draft_heads call: head inputs, both heads' logits, draft distributions, top-10 "
                         "(not in ms_per_step)"}
        del dh_w, dh_lg, dh_q
        # router + experts that feed the heads: 8 experts of the model's width (random weights)
        n_exp, d_ff = 8, d_model
        mo_u = torch.randn((dh_rows, d_model), device=dev, generator=gen).to(torch.bfloat16)
        mo_c = (torch.randn((n_exp, d_model), device=dev, generator=gen) * (1.5 / d_model ** 0.5)).to(torch.bfloat16)
        mo_w = [(torch.randn(shape, device=dev, generator=gen) * sc).to(torch.bfloat16)
                for shape, sc in (((n_exp, d_ff, d_model), d_model ** -0.5), ((n_exp, d_ff, d_model), d_model ** -0.5),
                                  ((n_exp, d_model, d_ff), d_ff ** -0.5))]
        mo_idx = torch.empty((dh_rows, 2), dtype=torch.int32, device=dev)
        mo_ws = torch.empty(jk.moe_experts_workspace(dh_rows, d_model, d_ff, n_exp), dtype=torch.uint8, device=dev)
        mo_call = jk.prepare_moe_experts(mo_u, mo_c, mo_w[0], mo_w[1], mo_w[2], dh_f, dh_s, mo_idx, None, mo_ws)
        def moe_pass():
            for _ in range(4):
                mo_call.launch()
        moe_pass()
        torch.cuda.synchronize()
        g_moe = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g_moe, stream=torch.cuda.Stream()):
            moe_pass()
        g_moe.replay()
        torch.cuda.synchronize()
        em0, em1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        em0.record()
        for _ in range(5):
            g_moe.replay()
        em1.record()
        torch.cuda.synchronize()
        mo_us = em0.elapsed_time(em1) * 1e3 / 20
        n_used = len(set(mo_idx.cpu().reshape(-1).tolist()))
        draft["moe_experts"] = {"us_per_call": round(mo_us, 1), "n_experts": n_exp, "experts_used": n_used,
                                "d_ff": d_ff,
                                "weight_stream_GBps": round(n_used * 3 * d_model * d_ff * 2 / (mo_us * 1e-6) / 1e9, 1),
                                "note": "one jk_moe_experts call: router, top-2, expert MLPs of the selected experts"}
        del mo_w
        # tree growth from the heads' candidates: one depth (5 frontier nodes per sequence), the cut to the
        # workload's tree size and the dense draft distributions for the acceptance call
        tg_front = 5
        tg_state = jk.TreeState(cfg.batch, 512)
        tg_tok = torch.randint(0, cfg.vocab, (cfg.batch * tg_front, 2, 10), dtype=torch.int32, device=dev, generator=gen)
        tg_p = torch.rand((cfg.batch * tg_front, 2, 10), device=dev, generator=gen).sort(dim=2, descending=True).values
        tg_root_tok, tg_root_p = tg_tok[: cfg.batch].contiguous(), tg_p[: cfg.batch].contiguous()
        tg_q = torch.rand((2 * cfg.batch * (1 + 2 * tg_front), cfg.vocab), device=dev, generator=gen)

        def tree_pass():
            tg_state.reset()
            fr = jk.tree_grow(tg_state, None, tg_root_tok, tg_root_p, tg_front, 0)
            for dpt in range(2):
                fr = jk.tree_grow(tg_state, fr, tg_tok, tg_p, tg_front, 2 * cfg.batch * (1 + dpt * tg_front))
            out = jk.tree_finalize(tg_state, cfg.n_tree)
            return jk.gather_draft_probs(tg_q, out[2])
        tree_pass()
        torch.cuda.synchronize()
        et0, et1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        et0.record()
        for _ in range(10):
            tree_pass()
        et1.record()
        torch.cuda.synchronize()
        eager_us = et0.elapsed_time(et1) * 1e3 / 10
        # the same round as one HIP graph (what a serving loop would replay): launch gaps instead of
        # Python and allocator time between the seven small kernels
        ref_q = tree_pass()
        torch.cuda.synchronize()
        g_tree = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g_tree, stream=torch.cuda.Stream()):
            graph_q = tree_pass()
        g_tree.replay()
        torch.cuda.synchronize()
        if not torch.equal(graph_q, ref_q):
            sys.exit("bench.py: the captured tree build differs from the eager one")
        et0.record()
        for _ in range(10):
            g_tree.replay()
        et1.record()
        torch.cuda.synchronize()
        draft["tree_build"] = {"us_per_round": round(et0.elapsed_time(et1) * 1e3 / 10, 1),
                               "us_per_round_eager": round(eager_us, 1), "depths": 3, "nodes_kept": cfg.n_tree,
                               "note": "3 jk_tree_grow + jk_tree_finalize + jk_gather_draft_probs; HIP-graph replay, "
                                       "and eager launches (which include torch's output allocations)"}
        del tg_q, graph_q, ref_q, g_tree

    # One whole round of the method as three HIP graphs (draft passes with the partial tree in the draft layer's
    # attention -> tree -> one attention call per target layer -> acceptance -> commit), random weights, the
    # shapes of this workload's model: what verify_steps_per_s has beside it on the draft side.
    whole_round = None
    if not args.no_extras and not args.no_draft_heads and cfg.mode == "sample" and cfg.dtype == "bf16" and cfg.tree_kind == "two_expert":
        from paper_2502_06282_amd import example_round
        d_model = cfg.n_q_heads * cfg.head_dim
        shape = dict(batch=cfg.batch, d_model=d_model, n_heads=cfg.n_q_heads, n_kv_heads=cfg.n_kv_heads,
                     head_dim=cfg.head_dim, d_ff=d_model, n_experts=8, vocab=cfg.vocab, depth=cfg.depth, top_k=cfg.topk,
                     width=cfg.frontier, n_tree=cfg.n_tree, prefix=cfg.prefix_len, target_layers=args.layers)
        rd = example_round.Round(seed=cfg.seed, **shape)
        whole_round = rd.time_phases(reps=10)
        whole_round.update(target_layers=args.layers, draft_passes=cfg.depth,
                           note="median of 10 replays; draft = per depth: reduction layer, q/k/v/o projections, attention "
                                "over the draft cache and the partial tree, router + experts, both heads, tree growth; "
                                "verify = the target layers' attention calls (the target's own projections and MLPs are "
                                "outside this library) + synthetic logits; refine = acceptance walk + commit of every layer")
        del rd
        torch.cuda.empty_cache()

    for _ in range(args.copy_calibration):
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
    torch.cuda.synchronize()

    # Which roof binds: the attention of one KV head is a dense contraction with T*G query rows per key;
    # above the ridge (peak flop/s / peak bytes/s = 312 flop/B) the matrix unit is the roof, below it HBM.
    intensity = flops_call / bytes_call
    kernel_name = ("tva_bf16_kernel" + ("" if plan["splits"] == 1 or plan["fused"] else " + tva_combine_bf16_kernel")
                   if cfg.dtype == "bf16" else "tva_f32_kernel + tva_combine_kernel")
    if intensity > MFMA_BF16_PEAK_TFLOPS * 1e3 / HBM_PEAK_GBPS and cfg.dtype == "bf16":
        roofline = {"bound": "mfma", "achieved": round(tflops, 1), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": round(tflops / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": MEASURED_TRAFFIC.get(cfg.name),
                    "secondary_hbm_GBps": round(gbps, 1)}
    else:
        roofline = {"bound": "hbm", "achieved": round(gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                    "frac": round(gbps / HBM_PEAK_GBPS, 4), "traffic": MEASURED_TRAFFIC.get(cfg.name),
                    "secondary_mfma_TFLOPs": round(tflops, 1)}
    roofline.update({"kernel": kernel_name + ": time per jk_tree_verify_attention call",
                     "algorithmic_bytes_per_launch": bytes_call, "algorithmic_flops_per_launch": int(flops_call),
                     "flop_per_byte": round(intensity, 1)})

    # Acceptance against the HBM roof: the dense bound (every logits row and, when sampling, every draft row
    # once), and - sampling reads rows lazily - the bytes the realised walk touched (from the oracle's walk of
    # the same inputs when the CPU leg ran, else None)
    acc_s = t_acc_ms * 1e-3
    rows = cfg.batch * (cfg.n_tree + 1)
    dense = rows * cfg.vocab * 4 + (cfg.batch * cfg.n_tree * cfg.vocab * 4 if mode == jk.JK_SAMPLE else 0)
    touched = dense if mode == jk.JK_GREEDY else (cpu or {}).get("accept_walk", {}).get("bytes_touched_by_the_walk")
    accept = {"us_per_call": round(t_acc_ms * 1e3, 2),
              "us_per_call_eight_in_one_graph_median_of_5": None if acc_b2b is None else round(acc_b2b, 2),
              "nodes_per_s": round(cfg.batch * cfg.n_tree / acc_s, 1),
              "accept_len": [int(v) for v in res[1].cpu().tolist()], "mode": cfg.mode,
              "dense_bytes": dense, "dense_bound_us": round(dense / (HBM_PEAK_GBPS * 1e9) * 1e6, 2),
              "bytes_touched": touched,
              "roofline": None if touched is None else
              {"bound": "hbm", "achieved": round(touched / acc_s / 1e9, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
               "frac": round(touched / acc_s / 1e9 / HBM_PEAK_GBPS, 4)},
              "deep_walk": deep}

    line = {
        "metric": "tree_verify_attention_hbm_GBps",
        "value": round(gbps, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if cfg.dtype == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: B{cfg.batch} Hq{cfg.n_q_heads} Hkv{cfg.n_kv_heads} D{cfg.head_dim} "
                               f"prefix{cfg.prefix_len} tree{cfg.n_tree} vocab{cfg.vocab} {cfg.mode}",
                   "layers": args.layers, "attention_calls_per_step": args.layers, "accept_calls_per_step": 1,
                   "launch": "eager" if args.no_graph else "hip_graph",
                   "kv_cache": f"paged, {args.paged} tokens per page" if args.paged else "contiguous",
                   "attention_plan": plan},
        "percent_of_hbm_peak": round(100.0 * gbps / HBM_PEAK_GBPS, 2),
        "verify_steps_per_s": round(1e3 / ms_per_step, 1),
        "attention_us_per_call": round(per_call_us, 3),
        "attention_TFLOPs": round(tflops, 1),
        "attention_timing": timing,
        "accept_us_per_call": round(t_acc_ms * 1e3, 2),
        "accept_nodes_per_s": round(cfg.batch * cfg.n_tree / acc_s, 1),
        "accept_len": [int(v) for v in res[1].cpu().tolist()],
        "accept": accept,
        "whole_round": whole_round,
        "stream_read_probe": probe,
        "commit_path": commit,
        "draft_heads": draft,
        "device_state": device_state(),
        "roofline": roofline,
    }
    if cpu is not None:
        line["cpu_baseline"] = cpu
    print(json.dumps(line))


if __name__ == "__main__":
    main()
