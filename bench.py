#!/usr/bin/env python3
"""Benchmark: tree decode attention over a prefix-shared paged KV cache on one MI355X.

A step is one spex_tree_decode_attention call on a fully built synthetic tree (page table ->
cached plan -> tree-walk kernel, or shared-prefix + suffix + merge kernels with --kernel-mode 2)
with all inputs resident in HBM.  Steps rotate over several identical trees in separate pools so
that no step finds its KV in the 256 MB last-level cache.  Prints one JSON line.
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
PAPER_CONTEXT = ("paper reports only end-to-end serving speedups (1.2-3x, up to 4.1x with MTP) on "
                 "NVIDIA A6000/A100; no attention-kernel number exists for this metric")
# The five configs of the metric (config 1 is the fp32 parity case) and the many-query workload.
PER_CONFIG = ["tiny_tree", "bfs_tot", "mcts_skewed", "spec_at_scale", "tot_with_drafts", "step_prefill"]


def source_sha16():
    """Hash of the sources that shape the kernels' memory traffic; a profile summary under
    profiles/ names the hash it was measured at."""
    import hashlib
    h = hashlib.sha256()
    for rel in ("paper_2605_10195_amd/csrc/kernels.hip", "paper_2605_10195_amd/csrc/planner.cpp"):
        with open(os.path.join(ROOT, rel), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def profiled_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` from the rocprofv3 --pmc summary profiles/<workload>_tree_walk.md
    (FETCH_SIZE + WRITE_SIZE, collected in runs of their own and scaled as the summary says).  The
    figure is reported only if the summary was made from the sources this run uses; else null."""
    path = os.path.join(ROOT, "profiles", f"{workload}_tree_walk.md")
    fields = {}
    try:
        with open(path) as f:
            for line in f:
                if line.startswith("    ") and ":" in line:
                    k, v = line.strip().split(":", 1)
                    fields[k.strip()] = v.strip()
    except OSError:
        return None, "no summary under profiles/ for this workload"
    if fields.get("kernel") != kernel or "traffic_bytes_per_launch" not in fields:
        return None, "the summary holds no traffic figure for this kernel"
    if fields.get("source_sha16") != source_sha16():
        return None, ("profiles/%s_tree_walk.md was measured at source hash %s, this run is %s"
                      % (workload, fields.get("source_sha16"), source_sha16()))
    return int(fields["traffic_bytes_per_launch"]), "profiles/%s_tree_walk.md" % workload


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="spec_at_scale",
                    choices=["tiny_tree", "bfs_tot", "mcts_skewed", "spec_at_scale", "tot_with_drafts",
                             "step_prefill", "dynamic_rebase", "dynamic_mcts"],
                    help="dynamic_rebase / dynamic_mcts: a breadth-first (REBASE widths, speculative "
                         "children verified at the level barrier) or depth-first (UCB descents, Alg. 1 "
                         "speculative expansions) search that grows while it is served, every decision "
                         "by the spex_sched_* primitives; --steps then counts decode iterations")
    ap.add_argument("--copies", type=int, default=0, help="rotating tree copies (0 = automatic)")
    ap.add_argument("--placement", default="random", choices=["random", "ascending"])
    ap.add_argument("--kv-pools", default="interleaved", choices=["interleaved", "separate"])
    ap.add_argument("--prefix-chunk", type=int, default=0)
    ap.add_argument("--suffix-chunk", type=int, default=0)
    ap.add_argument("--kernel-mode", type=int, default=0,
                    help="0 automatic, 2 shared-prefix + suffix + merge kernels, 3 tree-walk kernel")
    ap.add_argument("--walk-row-tiles", type=int, default=0)
    ap.add_argument("--walk-waves", type=int, default=0)
    ap.add_argument("--decode-iters", type=int, default=32,
                    help="after the timed steps: this many decode iterations (one token appended to "
                         "every branch with spex_tree_append_tokens, then attention) on one tree, "
                         "reported as decode_loop; 0 = skip")
    ap.add_argument("--token-trees", type=int, default=0,
                    help="verify a seeded draft token tree of this many tokens per branch (4-16, "
                         "tot_with_drafts only; visibility masks through "
                         "spex_tree_decode_attention_masked); 0 = the workload's causal drafts")
    ap.add_argument("--progress", action="store_true", help="print a line on stderr at every stage")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-per-config", action="store_true",
                    help="skip the short runs of the other configs that fill the per_config block")
    ap.add_argument("--cpu-sample-leaves", type=int, default=0)
    ap.add_argument("--calibrate", action="store_true",
                    help="also run one elementwise kernel that reads 1 GiB and writes 1 GiB, as the "
                         "known-size reference for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE")
    return ap.parse_args()


def cpu_baseline(wl, n_leaves, dev):
    """Time the oracle (its C form, oracle/attention_ref.c: materialise each branch's contiguous
    K/V, fp64 attention, requested nodes spread over the host's threads) on the first n_leaves
    requested nodes.  The seeded inputs are generated on `dev` and decoded to fp64 on the host before
    the clock starts."""
    import numpy as np

    import spex_workloads as sw
    from oracle import attention_c
    from oracle.adapters import OracleSink, queries_fp64

    leaves = wl.leaves[:n_leaves]
    q_lens = wl.q_lens[:n_leaves]
    _, parent, _ = wl.node_tokens()
    only = set()
    for u in leaves:
        while u != -1 and u not in only:
            only.add(u)
            u = parent[u]
    sink = OracleSink.for_workload(wl)
    sw.replay(wl, sink, device=dev, only_nodes=only)
    q = queries_fp64(sw.gen_queries(wl, device=dev)[:sum(q_lens)])
    masks = None if wl.draft_masks is None else [int(m) for m in wl.draft_masks[:sum(q_lens)]]
    threads = max(1, min(16, os.cpu_count() or 1))     # a one-GPU machine's share of the host
    t0 = time.perf_counter()
    out, _, info = attention_c.attention(sink.tree, leaves, q_lens, q, wl.sm_scale, draft_masks=masks,
                                         threads=threads)
    dt = time.perf_counter() - t0
    cpu_model = ""
    try:
        with open("/proc/cpuinfo") as f:
            cpu_model = next((ln.split(":", 1)[1].strip() for ln in f if ln.startswith("model name")), "")
    except OSError:
        pass
    busy = info["materialise_s"] + info["attention_s"]
    return dict(value=sum(q_lens) / dt, unit="query-tokens/s", cores=info["threads"], kind="oracle",
                cpu_model=cpu_model,
                sample=f"first {len(leaves)} of {len(wl.leaves)} requested branches "
                       f"({sum(q_lens)} query tokens): materialise each branch + fp64 attention in C, "
                       f"{info['threads']} threads over the branches, {dt:.2f} s wall",
                seconds=dt, materialise_share=info["materialise_s"] / busy if busy > 0 else 0.0,
                materialise_thread_seconds=info["materialise_s"],
                attention_thread_seconds=info["attention_s"]), out, leaves, q_lens


def decode_loop(tree, wl, q, out, lse, iters, dev):
    """The per-token loop of a step: every iteration appends one token to every requested branch
    (one spex_tree_append_tokens launch) and attends.  The new K/V are drawn before the timed
    region.  Reports wall time per iteration and how often the cached plan was patched / redone."""
    import torch

    import spex_workloads as sw
    import numpy as np
    nodes = np.asarray(sorted(set(wl.leaves)), dtype=np.int32)    # id arrays marshalled once, as a C caller holds them
    leaves = np.asarray(wl.leaves, dtype=np.int32)
    q_lens = np.asarray(wl.q_lens, dtype=np.int32)
    n = len(nodes)
    kv_torch = {"f32": torch.float32, "bf16": torch.bfloat16, "fp8_e4m3": torch.uint8}[wl.kv_dtype]
    ks = vs = None
    gen = torch.Generator(device=dev).manual_seed(7)
    src = torch.bfloat16 if wl.kv_dtype == "fp8_e4m3" else kv_torch
    k = (0.5 * torch.randn((n, wl.num_kv_heads, wl.head_dim), generator=gen, device=dev)).to(src)
    v = (0.5 * torch.randn((n, wl.num_kv_heads, wl.head_dim), generator=gen, device=dev)).to(src)
    quantize = wl.kv_dtype == "fp8_e4m3"        # bf16 tokens in, encoded by the append kernel
    if quantize:
        ks = torch.full((n, wl.num_kv_heads), 2.0 ** -7, dtype=torch.float32, device=dev)
        vs = ks.clone()
    counts = {0: 0, 1: 0, 2: 0}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(iters):
        tree.append_tokens(nodes, k, v, ks, vs, quantize=quantize)
        tree.decode_attention(leaves, q_lens, q, wl.sm_scale, out, lse, draft_masks=wl.draft_masks)
        counts[tree.last_launch_info()["plan_rebuilt"]] += 1
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / iters
    return dict(iterations=iters, ms_per_iteration=dt * 1e3, query_tokens_per_s=q.shape[0] / dt,
                plans_patched=counts[2], plans_redone=counts[1],
                note="append_tokens (fp8 pools: append_tokens_quantize, bf16 tokens encoded by the "
                     "append kernel) + decode_attention per iteration, one tree, KV of earlier "
                     "iterations may sit in the last-level cache; plans_patched counts iterations whose "
                     "cached plan was brought up to date (grown and started pages) inside the append "
                     "launch, plans_redone those that planned afresh")


def run_dynamic(args):
    """Decode iterations of a search whose trees change under it.  One iteration = one token for
    every generating branch (spex_tree_append_tokens) + decode attention over those branches;
    between iterations the scheduling primitives fork, speculate, verify, prune and terminate."""
    import numpy as np
    import torch

    import paper_2605_10195_amd as spex
    from paper_2605_10195_amd import binding as B
    from spex_workloads.dynamic import (DynamicConfig, DynamicShape, DynamicValues, LibrarySink,
                                        MctsConfig, MctsSpexDriver, RebaseSpexDriver)

    class Sched:
        rebase_widths = staticmethod(B.spex_sched_rebase_widths)
        allocate_budget = staticmethod(B.spex_sched_allocate_budget)
        early_termination = staticmethod(B.spex_sched_early_termination)
        ucb_select = staticmethod(B.spex_sched_ucb_select)
        dfs_speculate = staticmethod(B.spex_sched_dfs_speculate)
        make_tree = staticmethod(B.SearchTree)

    dev = "cuda:0"
    mcts = args.workload == "dynamic_mcts"
    if mcts:
        cfg = MctsConfig(n_queries=32, prompt=(512, 2048), branch=3, rollouts=24, c=0.6, step=(16, 160),
                         k_total=64, k_per_query=4, seed=17)
    else:
        cfg = DynamicConfig(n_queries=32, prompt=(512, 2048), budget=16, max_depth=6, step=(16, 160),
                            k_total=128, seed=11)
    shape = DynamicShape(32, 8, 128, 16, "bf16")
    n_pages = 65536
    order = np.random.default_rng(1000).permutation(n_pages).tolist()
    tree = spex.SpexTree(32, 8, 128, 16, "bf16", "bf16", num_pages=n_pages, device=dev, free_order=order,
                         interleave_kv=True, kernel_mode=args.kernel_mode,
                         walk_row_tiles=args.walk_row_tiles, walk_waves=args.walk_waves)
    b_tok = 2.0 * 8 * 128 * 2
    acc = dict(kv_tokens=0, peak_pages=0)

    class Sink(LibrarySink):
        def attend(self, nodes, iteration):
            super().attend(nodes, iteration)
            acc["kv_tokens"] += self.tree.last_launch_info()["kv_tokens"]
            acc["peak_pages"] = max(acc["peak_pages"], self.tree.stats()[1])

    sink = Sink(tree, shape, DynamicValues(shape, cfg.seed, dev, table_rows=8192), B.spex_tree_path_kv_bytes)
    driver = (MctsSpexDriver if mcts else RebaseSpexDriver)(cfg, sink, Sched)
    driver.run(args.warmup)               # starts the search and runs the warm-up iterations
    torch.cuda.synchronize()
    base = dict(driver.stats)
    states0, kv0, calls0 = dict(sink.plan_states), acc["kv_tokens"], dict(sink.call_seconds)
    tree.set_profiling(True)
    prof_ms, done = 0.0, 0
    t0 = time.perf_counter()
    while done < args.steps and driver.step():
        done += 1
        if done % 128 == 0:                      # the library keeps the last 256 calls
            prof_ms += float(tree.read_profile().sum())
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    prof_ms += float(tree.read_profile().sum())
    tokens = driver.stats["tokens"] - base["tokens"]
    kv_bytes = (acc["kv_tokens"] - kv0) * b_tok
    # how scattered the pages of a path are after all the forking and pruning
    live = sorted(driver.gen)[:64] if mcts else \
        [u for u, nd in driver.nodes.items() if nd.alive and not nd.children][:64]
    adjacent = total = 0
    for u in live:
        pages, _ = tree.path_pages(u)
        adjacent += sum(1 for a, b in zip(pages, pages[1:]) if b == a + 1)
        total += max(len(pages) - 1, 0)
    gbps = kv_bytes / (prof_ms * 1e-3) / 1e9 if prof_ms > 0 else 0.0
    result = {
        "metric": "tree decode-attn query-tokens/s + achieved HBM GB/s (unique KV bytes), 1 GPU",
        "value": tokens / wall, "unit": "query-tokens/s", "n_gpus": 1, "steps": done, "warmup": args.warmup,
        "ms_per_step": wall / max(done, 1) * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": args.workload, "queries": cfg.n_queries, "heads": [32, 8, 128],
                   "search": ({"branch": cfg.branch, "rollouts": cfg.rollouts, "c": cfg.c,
                               "k_per_query": cfg.k_per_query} if mcts else
                              {"budget": cfg.budget, "max_depth": cfg.max_depth}),
                   "prompt": list(cfg.prompt),
                   "step_tokens": list(cfg.step), "k_total": cfg.k_total, "pool_pages": n_pages,
                   "note": "a step is one decode iteration: append one token to every generating "
                           "branch, attention for those tokens, then the scheduling decisions"},
        "search": {k: (driver.stats[k] if k.startswith("max_") else driver.stats[k] - base.get(k, 0))
                   for k in driver.stats},
        "plans": {"cached": sink.plan_states[0] - states0[0], "fresh": sink.plan_states[1] - states0[1],
                  "patched": sink.plan_states[2] - states0[2]},
        "mean_branches_per_iteration": tokens / max(done, 1),
        "peak_pages_in_use": acc["peak_pages"],
        "adjacent_page_fraction_on_live_paths": adjacent / total if total else None,
        "roofline": {"bound": "hbm", "kernel": "spex_tree_walk_kernel", "achieved": gbps, "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": gbps / HBM_PEAK_GBPS, "traffic": None,
                     "bytes_per_launch": kv_bytes / max(done, 1), "ms_per_launch": prof_ms / max(done, 1),
                     "note": "kernel time from HIP events around every attention launch; bytes = "
                             "unique KV bytes of each launch's requested paths, summed"},
        "kernel_ms_share_of_wall": prof_ms / (wall * 1e3),
        "host_ms_per_step_in_library_calls": {k: (sink.call_seconds[k] - calls0[k]) / max(done, 1) * 1e3
                                              for k in sink.call_seconds},
        "cpu_baseline": None,
    }
    print(json.dumps(result, default=float))
    tree.close()


def measure(name, args, steps, warmup, decode_iters, cpu_sample, calibrate=False, progress=lambda m: None):
    """Build the synthetic trees of workload `name`, time `steps` decode-attention calls (plan
    cached, inputs resident in HBM), repeat them with HIP events around every kernel, and compare a
    sample of the output with the oracle.  Returns the result dictionary of one workload."""
    import numpy as np
    import torch

    import paper_2605_10195_amd as spex
    import spex_workloads as sw

    dev = "cuda:0"
    if args.token_trees and name == "tot_with_drafts":
        assert 1 <= args.token_trees <= 32
        wl = sw.tot_with_drafts(drafts=args.token_trees, token_trees=True)
    else:
        wl = sw.WORKLOADS[name]()
    if wl.draft_masks is not None:
        wl.draft_masks = np.asarray(wl.draft_masks, dtype=np.uint32)   # marshalled once, not per step
    n_pages = wl.peak_pages()
    unique_tokens = wl.unique_kv_tokens()
    unique_bytes = unique_tokens * wl.kv_bytes_per_token()
    copies = args.copies or max(1, min(8, int(2.5e9 // max(unique_bytes, 1)) + 1))
    if unique_bytes > 4e9:
        copies = args.copies or 1

    progress(f"workload {wl.name}: building {copies} tree(s), {n_pages} pages each")
    t_build = time.perf_counter()
    trees = []
    for c in range(copies):
        order = None
        if args.placement == "random":
            order = np.random.default_rng(1000 + c).permutation(n_pages).tolist()
        extra = len(set(wl.leaves)) * (decode_iters // wl.page_size + 2) if c == 0 else 0
        if order is not None and extra:
            order = order + list(range(n_pages, n_pages + extra))
        tree = spex.SpexTree(wl.num_q_heads, wl.num_kv_heads, wl.head_dim, wl.page_size, wl.q_dtype,
                             wl.kv_dtype, num_pages=n_pages + extra, device=dev, free_order=order,
                             prefix_chunk_pages=args.prefix_chunk, suffix_chunk_pages=args.suffix_chunk,
                             interleave_kv=args.kv_pools == "interleaved", kernel_mode=args.kernel_mode,
                             walk_row_tiles=args.walk_row_tiles, walk_waves=args.walk_waves)
        sw.replay(wl, tree, device=dev)
        trees.append(tree)
    q = sw.gen_queries(wl, device=dev)
    nq = q.shape[0]
    outs = [torch.empty((nq, wl.num_q_heads, wl.head_dim), dtype=torch.float32, device=dev)
            for _ in range(copies)]
    lses = [torch.empty((nq, wl.num_q_heads), dtype=torch.float32, device=dev) for _ in range(copies)]
    torch.cuda.synchronize()
    t_build = time.perf_counter() - t_build

    leaves_i32 = np.asarray(wl.leaves, dtype=np.int32)   # id arrays marshalled once, as a C caller holds them
    q_lens_i32 = np.asarray(wl.q_lens, dtype=np.int32)

    def step(i):
        c = i % copies
        trees[c].decode_attention(leaves_i32, q_lens_i32, q, wl.sm_scale, outs[c], lses[c],
                                  draft_masks=wl.draft_masks)

    progress("trees built; cold call")
    # cold call: plan build + upload + kernels
    t0 = time.perf_counter()
    step(0)
    torch.cuda.synchronize()
    cold_ms = (time.perf_counter() - t0) * 1e3
    info = trees[0].last_launch_info()
    for i in range(1, copies):
        step(i)
    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()

    progress("warm-up done; timed steps")
    # timed region: K steps, plan cached, no events
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall / steps * 1e3

    progress("timed steps done; steps with per-kernel events")
    # same K steps again with HIP events around every kernel (on the launch stream)
    for t in trees:
        t.set_profiling(True)
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    wall_prof = time.perf_counter() - t0
    prof = np.concatenate([t.read_profile() for t in trees], axis=0)
    for t in trees:
        t.set_profiling(False)
    k_ms = [float(x) for x in prof.mean(axis=0)]          # prefix, suffix, merge, tree-walk
    b_tok = wl.kv_bytes_per_token()
    kernels = {}
    walked = info["walk_row_tiles"] > 0
    for kname, ms, toks in (("prefix", k_ms[0], 0 if walked else info["prefix_tokens"]),
                            ("suffix", k_ms[1], 0 if walked else info["suffix_tokens"]),
                            ("walk", k_ms[3], info["kv_tokens"] if walked else 0)):
        gbps = toks * b_tok / (ms * 1e-3) / 1e9 if ms > 0 else 0.0
        kernels[kname] = dict(ms=float(ms), kv_tokens=int(toks), kv_bytes=float(toks * b_tok),
                              gbps=gbps, frac_hbm=gbps / HBM_PEAK_GBPS)
    part_bytes = 0 if walked else (info["partial_rows"] * (wl.head_dim + 2) * 4 +
                                   nq * wl.num_q_heads * (wl.head_dim + 1) * 4)
    kernels["merge"] = dict(ms=float(k_ms[2]), bytes=float(part_bytes),
                            gbps=part_bytes / (k_ms[2] * 1e-3) / 1e9 if k_ms[2] > 0 else 0.0)
    dominant = "walk" if walked else ("suffix" if k_ms[1] >= k_ms[0] else "prefix")
    dom = kernels[dominant]
    kernel_name = {"suffix": "spex_suffix_attn_kernel", "prefix": "spex_prefix_attn_kernel",
                   "walk": "spex_tree_walk_kernel"}[dominant]
    if wl.kv_dtype == "f32":
        kernel_name = "spex_generic_attn_kernel"
    traffic, traffic_source = profiled_traffic(wl.name, kernel_name)

    result = {
        "metric": "tree decode-attn query-tokens/s + achieved HBM GB/s (unique KV bytes), 1 GPU",
        "value": nq / (ms_per_step * 1e-3),
        "unit": "query-tokens/s",
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": {"f32": "f32", "bf16": "bf16", "fp8_e4m3": "fp8_e4m3 kv / bf16 q"}[wl.kv_dtype],
        "data": "synthetic",
        "config": {
            "workload": wl.name, "drafts_per_branch": max(wl.q_lens),
            "draft_visibility": "causal chain" if wl.draft_masks is None else "seeded token tree (masks)",
            "queries": wl.n_trees, "branches": len(wl.leaves),
            "query_tokens": nq, "heads": [wl.num_q_heads, wl.num_kv_heads, wl.head_dim],
            "page_size": wl.page_size, "unique_kv_tokens": unique_tokens,
            "unique_kv_bytes": unique_bytes, "flat_kv_bytes": wl.flat_kv_tokens() * b_tok,
            "tree_copies_rotated": copies, "page_placement": args.placement, "kv_pools": args.kv_pools,
            "prefix_chunk_pages": args.prefix_chunk, "suffix_chunk_pages": args.suffix_chunk,
            "kernels": "tree-walk" if walked else "shared-prefix + suffix + merge",
            "walk_row_tiles": int(info["walk_row_tiles"]), "walk_waves": int(info["walk_waves"]),
        },
        "hbm_gbps_unique_kv": unique_bytes / (ms_per_step * 1e-3) / 1e9,
        "hbm_frac_unique_kv": unique_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "roofline": {
            "bound": "hbm", "kernel": kernel_name, "achieved": dom["gbps"], "peak": HBM_PEAK_GBPS,
            "unit": "GB/s", "frac": dom["frac_hbm"],
            "traffic": traffic, "traffic_source": traffic_source,
            "bytes_per_launch": dom["kv_bytes"], "ms_per_launch": dom["ms"],
        },
        "kernels": kernels,
        "kernels_ms_sum": float(sum(k_ms)),
        "ms_per_step_profiled": wall_prof / steps * 1e3,
        "cold_call_ms": cold_ms,
        "launch": {k: int(v) for k, v in info.items()},
        "build_seconds": t_build,
    }

    sample_out = outs[0].clone()          # the decode loop below reuses outs[0] on a grown tree
    progress("per-kernel steps done; decode loop / calibration / cpu baseline")
    if decode_iters > 0:
        result["decode_loop"] = decode_loop(trees[0], wl, q, outs[0], lses[0], decode_iters, dev)

    if calibrate:
        ref_in = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        ref_out = torch.empty_like(ref_in)
        torch.cuda.synchronize()
        torch.add(ref_in, 1.0, out=ref_out)
        torch.cuda.synchronize()
        del ref_in, ref_out

    for t in trees:
        t.close()
    del trees, outs, lses
    torch.cuda.empty_cache()

    if cpu_sample > 0:
        base, ref_out, leaves, q_lens = cpu_baseline(wl, cpu_sample, dev)
        got = sample_out[:ref_out.shape[0]].cpu().numpy().astype(np.float64)
        d = got - ref_out
        base["gpu_vs_oracle_max_abs"] = float(np.max(np.abs(d)))
        base["gpu_vs_oracle_rel_l2"] = float(np.linalg.norm(d) / np.linalg.norm(ref_out))
        rows_d = np.linalg.norm(d.reshape(-1, d.shape[-1]), axis=1)
        rows_r = np.linalg.norm(ref_out.reshape(-1, d.shape[-1]), axis=1)
        base["gpu_vs_oracle_worst_row_rel_l2"] = float(np.max(rows_d / np.maximum(rows_r, 1e-300)))
        result["cpu_baseline"] = base
    else:
        result["cpu_baseline"] = None

    if wl.name == "step_prefill":
        # many queries per branch: the contraction, not the KV stream, bounds this workload.
        # flops = 4 * D per (query token, query head, visible KV token): QK^T and PV, 2 each
        visible = 0
        for leaf, ql in zip(wl.leaves, wl.q_lens):
            T = wl.path_tokens(leaf)
            visible += ql * (T - ql) + ql * (ql + 1) // 2
        flops = 4.0 * wl.head_dim * wl.num_q_heads * visible
        tfs = flops / (dom["ms"] * 1e-3) / 1e12
        result["roofline"] = {"bound": "mfma", "kernel": kernel_name, "achieved": tfs,
                              "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": tfs / MFMA_BF16_PEAK_TFLOPS,
                              "traffic": traffic, "traffic_source": traffic_source,
                              "flops_per_launch": flops, "ms_per_launch": dom["ms"],
                              "hbm_gbps_unique_kv": dom["gbps"]}
    return result


# requested branches the oracle is timed on (about 10-30 s of host work each on 16 threads)
CPU_SAMPLE = {"tiny_tree": 4, "bfs_tot": 512, "mcts_skewed": 1105, "spec_at_scale": 2048,
              "tot_with_drafts": 512, "tot_with_drafts_token_trees": 512, "step_prefill": 64}
# ... and on which the short per-config runs compare the GPU output with it
PARITY_SAMPLE = {"tiny_tree": 4, "bfs_tot": 128, "mcts_skewed": 256, "spec_at_scale": 256,
                 "tot_with_drafts": 64, "step_prefill": 8}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path shards by tree or by KV head "
              "without any exchange between GPUs); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.workload in ("dynamic_rebase", "dynamic_mcts"):
        run_dynamic(args)
        return

    def progress(msg):
        if args.progress:
            print(f"[bench {time.strftime('%H:%M:%S')}] {msg}", file=sys.stderr, flush=True)

    key = args.workload + ("_token_trees" if args.token_trees and args.workload == "tot_with_drafts" else "")
    cpu_sample = 0 if args.no_cpu_baseline else (args.cpu_sample_leaves or CPU_SAMPLE[key])
    result = measure(args.workload, args, args.steps, args.warmup, args.decode_iters, cpu_sample,
                     calibrate=args.calibrate, progress=progress)
    result["paper_context"] = PAPER_CONTEXT
    result["source_sha16"] = source_sha16()

    if not args.no_per_config:
        # every config of the metric in the same line: short runs of the others, each with its
        # roofline fraction and its error against the oracle on a sample of branches
        per = {}
        for name in PER_CONFIG:
            if name == args.workload:
                r = result
            else:
                progress(f"per-config run: {name}")
                r = measure(name, args, min(args.steps, 50), min(args.warmup, 10), 0,
                            0 if args.no_cpu_baseline else PARITY_SAMPLE[name], progress=progress)
            rl, cb = r["roofline"], r["cpu_baseline"]
            per[name] = {
                "ms_per_step": r["ms_per_step"], "query_tokens_per_s": r["value"],
                "kernel": rl["kernel"], "kernel_ms": rl["ms_per_launch"], "bound": rl["bound"],
                "frac": rl["frac"], "achieved": rl["achieved"], "unit": rl["unit"],
                "hbm_frac_unique_kv_wall": r["hbm_frac_unique_kv"],
                "kernels": r["config"]["kernels"], "tree_copies_rotated": r["config"]["tree_copies_rotated"],
                "steps": r["steps"],
                "parity": None if cb is None else {
                    "branches": cb["sample"].split(" requested")[0],
                    "max_abs": cb["gpu_vs_oracle_max_abs"], "rel_l2": cb["gpu_vs_oracle_rel_l2"],
                    "worst_row_rel_l2": cb["gpu_vs_oracle_worst_row_rel_l2"]},
            }
        result["per_config"] = per
    progress("done")
    print(json.dumps(result, default=float))


if __name__ == "__main__":
    main()
