#!/usr/bin/env python3
"""Benchmark of the Talon hot path on one MI355X.

One step = tree init + the whole budget-driven expansion loop (vocab scan + budget
selection per layer) + tree-mask build + one tree-attention call, for one batch of
synthetic inputs already resident in HBM.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config c2]

The default workload is the Llama-3-8B-shaped configuration the headline metric is quoted
on.  Inputs rotate over several independently generated pools and KV buffers so that
consecutive steps do not find their rows in the 256 MB Infinity Cache.
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

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 MFMA


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", default="c2", help="c1..c5 (default c2: the headline workload)")
    ap.add_argument("--slots", type=int, default=0, help="rotating input sets (0 = enough to exceed 512 MB)")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying HIP graphs")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-c3", action="store_true", help="leave the Qwen3-8B x4 block out of the default line")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run plain device copies of 1 GiB (reads 1 GiB, writes 1 GiB each): the "
                         "reference that scales the FETCH_SIZE / WRITE_SIZE counters of a --pmc run")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="budget for the oracle timing sample")
    ap.add_argument("--probes", action="store_true",
                    help="cycles per instruction of the attention step's instruction mixes (one and two wavefronts "
                         "per SIMD) and the rate of direct-to-LDS tile loads per compute unit")
    ap.add_argument("--attainable", action="store_true",
                    help="only run the library's two probes: a streaming read of 1 GiB and 512 MiB buffers (cold) "
                         "and a register-resident bf16 MFMA loop; prints the rates they reach")
    ap.add_argument("--cap", type=int, default=0,
                    help="per-row candidate cap k (default: the config's K).  A cap >= N - 1 gives the tree of "
                         "Alg. 2 as printed (every token of every parent in the pool); the first layer stays Top-K")
    ap.add_argument("--accept", action="store_true",
                    help="also time the greedy verification outcome that follows a step (target argmax over every "
                         "tree node, acceptance walk, accepted-path KV compaction) on synthetic target logits")
    ap.add_argument("--sweep", action="store_true",
                    help="budget N, threshold mu and top-K-initialised layers swept on the c2 shape, with the "
                         "bookkeeping of Sec. 5.3 / App. C per variant (tree size, depth, rows scanned, accepted length)")
    ap.add_argument("--scan-grid", action="store_true",
                    help="the vocabulary scan alone (talon_expand_layer) on the c5 pool with every node a frontier row: "
                         "HBM rate against the number of rows and the per-row k")
    ap.add_argument("--zipf-grid", action="store_true",
                    help="only run the paper's tree-construction micro-benchmark shape (App. E.6): latency of one "
                         "layer expansion over K parents with Zipf rows, exponent x vocabulary grid, 20 warm-ups and "
                         "100 timed runs, for the adaptive gate (Alg. 2) and the static top-K of the pool (Alg. 1)")
    ap.add_argument("--literal", action="store_true",
                    help="time the expansion with the uncapped candidate pool (talon_tree_init + talon_expand_literal "
                         "+ talon_build_tree_mask) beside the capped single launch on the same inputs, and report how "
                         "the two trees differ")
    ap.add_argument("--layerwise", action="store_true",
                    help="also time the expansion layer by layer (one fused scan+selection launch per layer, "
                         "talon_expand_select_layer) and report rows, duration and read bandwidth of each layer")
    return ap.parse_args()


class Slot:
    """One set of inputs (logits pool, Q/K/V) on the device, with the tree state and mask its
    steps write (so that what every slot's last step produced can be checked after timing)."""

    def __init__(self, cfg, seed, torch, H, T=None):
        import numpy as np
        from workloads import attention_inputs
        seeds = [seed] * cfg.B
        self.seed = seed
        pool = H.build_pool(cfg, seeds)
        self.logits = H.to_device_logits(pool)
        xs = [attention_inputs(cfg, seed, b) for b in range(cfg.B)]
        self.q = H.bf16_to_device(np.stack([x["q"] for x in xs]))
        self.kp = H.bf16_to_device(np.stack([x["k_prefix"] for x in xs]))
        self.vp = H.bf16_to_device(np.stack([x["v_prefix"] for x in xs]))
        self.kt = H.bf16_to_device(np.stack([x["k_tree"] for x in xs]))
        self.vt = H.bf16_to_device(np.stack([x["v_tree"] for x in xs]))
        self.graph = None
        self.graph_layers = None
        if T is not None:
            self.st = T.TreeState(cfg.B, cfg.N)
            self.mask = torch.zeros(cfg.B, self.st.N_pad, self.st.N_pad // 64, dtype=torch.int64, device="cuda")
        self.n_expected = None


def check_slots(T, slots, used, where):
    """Every slot's last step must have ended normally and built the tree its warm-up built: a
    launch that gave up its bounded wait (ABORTED) or met a bad row must not be timed as a step."""
    bad = T.TALON_STATUS_ABORTED | T.TALON_STATUS_BAD_ROW
    for i in sorted(set(used)):
        s = slots[i]
        status = s.st.status.cpu().numpy()
        n = s.st.n_nodes.cpu().numpy()
        if (status & bad).any() or not ((status & 3) != 0).all():
            print("bench.py: %s: slot %d ended with status %s" % (where, i, status.tolist()), file=sys.stderr)
            sys.exit(3)
        if s.n_expected is not None and n.tolist() != s.n_expected:
            print("bench.py: %s: slot %d built trees of %s nodes, warm-up built %s" %
                  (where, i, n.tolist(), s.n_expected), file=sys.stderr)
            sys.exit(3)


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding or collectives are part of it); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    from workloads import CONFIGS
    cfg = CONFIGS[args.config.lower()]
    plain = not (args.copy_calibration or args.attainable or args.probes or args.zipf_grid or args.scan_grid
                 or args.sweep or args.literal)
    # The oracle's timing runs first, in forked worker processes, before this process touches
    # the GPU (a process that has initialised the GPU must not be forked into workers).
    cpu = None
    if plain and not args.no_cpu_baseline:
        cpu = cpu_baseline(cfg, args.cpu_seconds)

    import numpy as np
    import torch
    import paper_2601_07353_amd as T
    import workloads as H

    T.load_library()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": {"bytes_read": 1 << 30, "bytes_written": 1 << 30, "copies": 10}}))
        return

    if args.probes:
        print(json.dumps({"probes": probes(T, torch)}))
        return
    if args.attainable:
        print(json.dumps({"attainable": attainable(T, torch)}))
        return
    if args.zipf_grid:
        print(json.dumps({"zipf_grid": zipf_grid(T, torch, np, H)}))
        return
    if args.scan_grid:
        print(json.dumps({"scan_grid": scan_grid(T, torch, np, H)}))
        return
    if args.sweep:
        print(json.dumps({"sweep": variant_sweep(T, torch, np, H, args.steps)}))
        return
    if args.literal:
        print(json.dumps({"literal": literal_timing(T, torch, np, H, cfg, args.steps, args.slots or 2)}))
        return

    r = run_workload(T, torch, np, H, cfg, args, args.steps, args.warmup)
    result = {
        "metric": "tree expand+verify steps/s", "value": r["steps_per_s"], "unit": "steps/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": r["ms_per_step"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if cfg.logits_dtype == "bf16" else "f32",
        "data": "synthetic",
        "config": r["config"],
        "roofline": r["roofline"],
        "kernels": r["kernels"],
        "latency": r["latency"],
        "per_layer_launches": r["per_layer_launches"],
    }
    for key in ("accept", "layers"):
        if key in r:
            result[key] = r[key]
    # The second 8B-shaped configuration (Qwen3-8B x4: wide layers, where the bandwidth and
    # matrix-core fractions mean something) rides along on the default line.
    if cfg.name == CONFIGS["c2"].name and not args.no_c3:
        c3 = run_workload(T, torch, np, H, CONFIGS["c3"], args, min(args.steps, 100), min(args.warmup, 10), extras=False)
        result["c3"] = {"workload": c3["config"]["workload"], "steps_per_s": c3["steps_per_s"],
                        "ms_per_step": c3["ms_per_step"], "steps": c3["steps"], "config": c3["config"],
                        "expand_tree_kernel": c3["kernels"]["expand_tree_kernel"],
                        "tree_attention": c3["kernels"]["tree_attention"],
                        "per_layer_launches": c3["per_layer_launches"]}
    if cpu is not None:
        result["cpu_baseline"] = cpu
    print(json.dumps(result))


def run_workload(T, torch, np, H, cfg, args, steps, warmup, extras=True):
    """Times `steps` whole steps of one configuration; returns the figures of the bench line."""
    dev = torch.device("cuda:0")
    elem = cfg.elem_bytes
    pool_bytes = cfg.B * cfg.N_pad * cfg.V * elem
    kv_bytes = 2 * cfg.B * cfg.L * cfg.Hkv * cfg.Dh * 2
    n_slots = args.slots or max(2, min(32, int(np.ceil(512e6 / (pool_bytes + kv_bytes)))))
    slots = [Slot(cfg, cfg.seed + 1000 * i, torch, H, T) for i in range(n_slots)]

    cap = args.cap or cfg.K
    N_pad = slots[0].st.N_pad
    cand = T.Candidates(cfg.B, N_pad, cap)
    dt = T.TALON_DTYPE_F32 if cfg.logits_dtype == "f32" else T.TALON_DTYPE_BF16
    ws_expand = T.make_expand_workspace(cfg.B, N_pad, cfg.V, cap, dt)
    roots = torch.from_numpy(H.root_tokens(cfg)).cuda()
    out = torch.zeros(cfg.B, N_pad, cfg.Hq, cfg.Dh, dtype=torch.bfloat16, device=dev)
    plen = torch.full((cfg.B,), cfg.L, dtype=torch.int32, device=dev)
    nb = T.talon_tree_attention_workspace_bytes(cfg.B, N_pad, cfg.Hq, cfg.Hkv, cfg.Dh, cfg.L)
    ws_attn = torch.empty(max(nb, 256), dtype=torch.uint8, device=dev)
    depth_cap = min(cfg.Dmax, cfg.N - 1)

    def expand(s):   # tree init, the whole loop of Alg. 2 and the ancestor mask: one launch
        T.talon_build_tree(roots, s.logits, s.st, cap, cfg.mu, cfg.K, 1, cfg.Dmax, cand, ws_expand, mask=s.mask)

    def attention(s):
        T.talon_tree_attention(s.q, s.kp, s.vp, s.kt, s.vt, s.mask, s.st.n_nodes, plen, cfg.L, out, None, ws_attn)

    def step(s):
        expand(s)
        attention(s)

    def step_per_layer(s):   # what a serving loop can call between draft passes: one launch per layer
        T.talon_tree_init(s.st, roots)
        for d in range(depth_cap):
            T.talon_expand_select_layer(s.logits, s.st, cap, cfg.mu, cfg.K, 1, cfg.Dmax, cand, ws_expand, layer=d)
        T.talon_build_tree_mask(s.st, s.mask)
        attention(s)

    # ---- warmup (also records the per-slot work: rows scanned, attention FLOPs)
    rows_scanned, attn_flops, n_nodes_mean = [], [], []
    for i in range(max(warmup, n_slots)):
        s = slots[i % n_slots]
        step(s)
        if i < n_slots:
            torch.cuda.synchronize()
            n = s.st.n_nodes.cpu().numpy().astype(np.int64)
            fc = s.st.frontier_count.cpu().numpy().astype(np.int64)
            depth = s.st.depth.cpu().numpy()
            s.n_expected = n.tolist()
            rows_scanned.append(int((n - fc).sum()))
            keys = sum(int((cfg.L + depth[b, :n[b]] + 1).sum()) for b in range(cfg.B))
            attn_flops.append(4.0 * cfg.Hq * cfg.Dh * keys)
            n_nodes_mean.append(float(n.mean()))
    torch.cuda.synchronize()
    check_slots(T, slots, range(n_slots), "warm-up")

    use_graph = not args.no_graph
    if use_graph:
        for s in slots:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                step(s)
            s.graph = g
        for s in slots:
            s.graph.replay()
        torch.cuda.synchronize()

    # ---- timed region: exactly K steps
    used = [i % n_slots for i in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in used:
        s = slots[i]
        if use_graph:
            s.graph.replay()
        else:
            step(s)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / steps
    steps_per_s = steps / (t1 - t0)
    check_slots(T, slots, used, "timed region")

    # ---- the same steps with one launch per layer (tree init, Dmax fused scan + selection
    # launches, mask, attention), as one HIP graph per slot
    per_layer = None
    if use_graph:
        for s in slots:
            step_per_layer(s)
        torch.cuda.synchronize()
        check_slots(T, slots, range(n_slots), "per-layer launches, eager")
        for s in slots:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                step_per_layer(s)
            s.graph_layers = g
        for s in slots:
            s.graph_layers.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in used:
            slots[i].graph_layers.replay()
        torch.cuda.synchronize()
        dt_s = time.perf_counter() - t0
        check_slots(T, slots, used, "per-layer launches")
        per_layer = {"ms_per_step": dt_s * 1e3 / steps, "steps_per_s": steps / dt_s,
                     "launches_per_step": 2 + depth_cap + (2 if nb > 256 else 1),
                     "what": "talon_tree_init + %d x talon_expand_select_layer (one launch each: the scan with the "
                             "selections in its tail; layers after a tree is complete find no work) + "
                             "talon_build_tree_mask + talon_tree_attention, one HIP graph per step" % depth_cap}

    # ---- kernel timing region: the same K steps launched eagerly, with HIP events (on the
    # launch stream) around the expansion launch (one per step: the kernel walks all layers;
    # recorded by the library's measurement hook inside talon_build_tree) and around the
    # tree-attention call.
    layers = 1
    ev_attn = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    T.talon_profile_scan_launches(True)
    for k_, i in enumerate(used):
        s = slots[i]
        expand(s)
        e0, e1 = ev_attn[k_]
        e0.record(); attention(s); e1.record()
    torch.cuda.synchronize()
    scan_us, n_rec = T.talon_profile_read(steps * layers)
    T.talon_profile_scan_launches(False)
    assert n_rec == steps * layers, (n_rec, steps, layers)
    check_slots(T, slots, used, "kernel timing region")
    scan_ms_step = float(np.sum(scan_us)) * 1e-3 / steps
    scan_ms_launch = scan_ms_step / layers
    attn_all = [e0.elapsed_time(e1) for e0, e1 in ev_attn]
    attn_ms = float(np.mean(attn_all))
    # one step at a time (a graph replay between two events, the device idle before it): the
    # latency a single request sees, as mean and median beside the back-to-back rate above
    lat = []
    if use_graph and extras:
        for i in used[:100]:
            s = slots[i]
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record(); s.graph.replay(); e1.record()
            torch.cuda.synchronize()
            lat.append(e0.elapsed_time(e1) * 1e3)
    latency = {"expand_launch_us_mean": float(np.mean(scan_us)), "expand_launch_us_p50": float(np.median(scan_us)),
               "attention_us_mean": attn_ms * 1e3, "attention_us_p50": float(np.median(attn_all)) * 1e3,
               "single_step_us_mean": float(np.mean(lat)) if lat else None,
               "single_step_us_p50": float(np.median(lat)) if lat else None}

    mean_rows = float(np.mean([rows_scanned[u] for u in used]))
    mean_flops = float(np.mean([attn_flops[u] for u in used]))
    scan_bytes = mean_rows * cfg.V * elem
    attn_bytes = (2.0 * cfg.B * cfg.L * cfg.Hkv * cfg.Dh * 2 +
                  2.0 * float(np.mean(n_nodes_mean)) * cfg.B * (cfg.Hq + cfg.Hkv) * cfg.Dh * 2)

    scan_gbps = scan_bytes / (scan_ms_step * 1e-3) / 1e9
    attn_tflops = mean_flops / (attn_ms * 1e-3) / 1e12
    kernels = {
        "expand_tree_kernel": {"launches_per_step": layers, "ms_per_step": scan_ms_step, "ms_per_launch": scan_ms_launch,
                               "rows_scanned_per_step": mean_rows, "bytes_per_step": scan_bytes,
                               "GBps": scan_gbps, "frac_of_hbm_peak": scan_gbps / HBM_PEAK_GBS},
        "tree_attention": {"ms": attn_ms, "flops": mean_flops, "bytes": attn_bytes,
                           "TFLOPs": attn_tflops, "frac_of_mfma_peak": attn_tflops / MFMA_BF16_PEAK_TFLOPS},
    }
    traffic = read_traffic(cfg.name)
    traffic_source = ("profiles/hbm_traffic_%s.txt: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command, "
                      "scaled by a plain 1 GiB copy; a committed summary, not counted in this run" % cfg.name)
    if scan_ms_step >= attn_ms:
        # dominant kernel of the step: the vocab scan (HBM-bound: every logit is read once)
        ach = scan_bytes / layers / (scan_ms_launch * 1e-3) / 1e9
        roofline = {"kernel": "expand_tree_kernel", "bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": ach / HBM_PEAK_GBS, "traffic": traffic.get("expand_tree_kernel"),
                    "traffic_source": traffic_source,
                    "launches_per_step": layers, "avg_launch_us": scan_ms_launch * 1e3,
                    "algorithmic_bytes_per_launch": scan_bytes / layers}
    else:
        ach = mean_flops / (attn_ms * 1e-3) / 1e12
        roofline = {"kernel": "tree_attention_kernel", "bound": "mfma", "achieved": ach,
                    "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": ach / MFMA_BF16_PEAK_TFLOPS,
                    "traffic": traffic.get("tree_attention_kernel"), "traffic_source": traffic_source,
                    "avg_launch_us": attn_ms * 1e3, "algorithmic_flops_per_launch": mean_flops}

    r = {"steps_per_s": steps_per_s, "ms_per_step": ms_per_step, "steps": steps,
         "config": {"workload": cfg.name, "B": cfg.B, "vocab": cfg.V, "K": cfg.K, "N": cfg.N, "Dmax": cfg.Dmax,
                    "mu": cfg.mu, "row_cap": cap, "Hq": cfg.Hq, "Hkv": cfg.Hkv, "Dh": cfg.Dh, "prefix_len": cfg.L,
                    "input_slots": n_slots, "hip_graph": use_graph},
         "roofline": roofline, "kernels": kernels, "latency": latency, "per_layer_launches": per_layer}
    st = slots[(steps - 1) % n_slots].st
    if args.accept and extras:
        r["accept"] = accept_outcome(T, torch, np, cfg, slots, st, steps, elem)
    if args.layerwise and extras:
        r["layers"] = layerwise(T, torch, np, cfg, slots, st, cand, ws_expand, roots, steps, elem)
    return r


def accept_outcome(T, torch, np, cfg, slots, st, steps, elem):
    """The calls that follow a step at temperature 0, timed as one HIP graph per replay on the
    tree the last step left in `st`: talon_target_argmax (one vocabulary scan with k = 1 over
    every tree node: n * V * sizeof(dtype) bytes per sequence, HBM-bound), talon_greedy_accept,
    talon_compact_kv.  Target logits: random rows of the draft pools of other slots (any row
    serves: the scan's cost does not depend on the values)."""
    dt = T.TALON_DTYPE_F32 if cfg.logits_dtype == "f32" else T.TALON_DTYPE_BF16
    ws = T.make_verify_workspace(cfg.B, st.N_pad, cfg.V, dt)
    dev = "cuda"
    tgt = torch.zeros(cfg.B, st.N_pad, dtype=torch.int32, device=dev)
    prob = torch.zeros(cfg.B, st.N_pad, dtype=torch.float32, device=dev)
    sstat = torch.zeros(cfg.B, dtype=torch.int32, device=dev)
    path = torch.zeros(cfg.B, st.N_pad, dtype=torch.int32, device=dev)
    alen = torch.zeros(cfg.B, dtype=torch.int32, device=dev)
    bonus = torch.zeros(cfg.B, dtype=torch.int32, device=dev)
    cap = cfg.L + st.N_pad
    kp = torch.zeros(cfg.B, cap, cfg.Hkv, cfg.Dh, dtype=torch.bfloat16, device=dev)
    vp = torch.zeros_like(kp)
    plen = torch.full((cfg.B,), cfg.L, dtype=torch.int32, device=dev)
    new_plen = torch.zeros(cfg.B, dtype=torch.int32, device=dev)

    def outcome(s):
        T.talon_target_argmax(s.logits, st, tgt, prob, sstat, ws)
        T.talon_greedy_accept(st, tgt, sstat, path, alen, bonus)
        T.talon_compact_kv(s.kt, s.vt, path, alen, plen, new_plen, kp, vp)

    graphs = []
    for s in slots:
        outcome(s)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            outcome(s)
        graphs.append(g)
    for g in graphs:
        g.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        graphs[i % len(graphs)].replay()
    torch.cuda.synchronize()
    us = (time.perf_counter() - t0) * 1e6 / steps
    rows = float(st.n_nodes.sum().item())
    by = rows * cfg.V * elem
    return {"us_per_call": us, "target_rows": rows, "bytes": by, "GBps": by / (us * 1e-6) / 1e9,
            "accepted_mean": float(alen.float().mean().item())}


def scan_grid(T, torch, np, H):
    """talon_expand_layer alone on the c5 pool (16 sequences, 151936 bf16 logits per row), the
    frontier set by hand to the first 32 / 128 / 256 nodes of every sequence, k = 1, 8, 16: what
    the one-pass softmax + top-k scan sustains when nothing else is in the launch.  Two copies
    of the 1.24 GB pool alternate, so no launch finds its rows in a cache."""
    from workloads import CONFIGS
    cfg = CONFIGS["c5"]
    dev = H.to_device_logits(H.build_pool(cfg, [cfg.seed] * cfg.B))
    other = dev.clone()
    out = []
    for rows_per_seq in (256, 128, 32):
        for k in (1, 8, 16):
            st = T.TreeState(cfg.B, cfg.N)
            st.n_nodes.fill_(rows_per_seq); st.frontier_begin.fill_(0); st.frontier_count.fill_(rows_per_seq)
            st.status.fill_(0)
            cand = T.Candidates(cfg.B, st.N_pad, k)
            ws = T.make_expand_workspace(cfg.B, st.N_pad, cfg.V, k, T.TALON_DTYPE_BF16)
            for _ in range(2):
                T.talon_expand_layer(dev, st, k, cand, ws)
                T.talon_expand_layer(other, st, k, cand, ws)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            reps = 10
            e0.record()
            for i in range(reps):
                T.talon_expand_layer(dev if i % 2 == 0 else other, st, k, cand, ws)
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / reps
            by = cfg.B * rows_per_seq * cfg.V * 2
            out.append({"rows": cfg.B * rows_per_seq, "k": k, "us": us, "bytes": by, "GBps": by / us / 1e3,
                        "frac_of_8TBps": by / us / 1e3 / HBM_PEAK_GBS})
    return out


def variant_sweep(T, torch, np, H, steps):
    """The knobs of Alg. 2 as the paper varies them (budget N, Table 5; threshold mu, Fig. 6; number
    of top-K-initialised layers, Table 6), on the c2 shape: whole steps (talon_build_tree +
    talon_tree_attention) replayed as HIP graphs over rotating inputs, then the temperature-0
    outcome on synthetic target rows (the draft row plus noise: a stand-in for a target model that
    mostly agrees with its draft) for the accepted length.  Per variant: steps/s, tree size n,
    depth reached, rows scanned R, accepted draft tokens and tau = accepted + 1 (the bonus token)."""
    import dataclasses
    from workloads import CONFIGS, target_logits_pool
    base = dataclasses.replace(CONFIGS["c2"], N=96)          # pools hold rows for the largest budget
    n_slots = 12
    slots, targets = [], []
    for i in range(n_slots):
        sl = Slot(base, base.seed + 1000 * i, torch, H)
        slots.append(sl)
        targets.append(H.to_device_logits(target_logits_pool(base, sl.seed)))
    dev = "cuda"
    dt = T.TALON_DTYPE_BF16
    variants = [dict(N=N, mu=0.03, init_layers=1) for N in (32, 48, 60, 64, 80, 96)]
    variants += [dict(N=60, mu=mu, init_layers=1) for mu in (0.003, 0.01, 0.1, 0.3)]
    variants += [dict(N=60, mu=0.03, init_layers=k) for k in (0, 2, 3)]
    rows_out = []
    for v in variants:
        cfg = dataclasses.replace(base, N=v["N"], mu=v["mu"])
        st = T.TreeState(1, cfg.N)
        Np = st.N_pad
        cand = T.Candidates(1, Np, cfg.K)
        ws = T.make_expand_workspace(1, Np, cfg.V, cfg.K, dt)
        vws = T.make_verify_workspace(1, Np, cfg.V, dt)
        roots = torch.from_numpy(H.root_tokens(cfg)).cuda()
        mask = torch.zeros(1, Np, Np // 64, dtype=torch.int64, device=dev)
        out = torch.zeros(1, Np, cfg.Hq, cfg.Dh, dtype=torch.bfloat16, device=dev)
        plen = torch.full((1,), cfg.L, dtype=torch.int32, device=dev)
        nb = T.talon_tree_attention_workspace_bytes(1, Np, cfg.Hq, cfg.Hkv, cfg.Dh, cfg.L)
        wa = torch.empty(max(nb, 256), dtype=torch.uint8, device=dev)
        tgt = torch.zeros(1, Np, dtype=torch.int32, device=dev)
        prob = torch.zeros(1, Np, dtype=torch.float32, device=dev)
        sstat = torch.zeros(1, dtype=torch.int32, device=dev)
        path = torch.zeros(1, Np, dtype=torch.int32, device=dev)
        alen = torch.zeros(1, dtype=torch.int32, device=dev)
        bonus = torch.zeros(1, dtype=torch.int32, device=dev)

        def step(sl):
            T.talon_build_tree(roots, sl.logits, st, cfg.K, cfg.mu, cfg.K, v["init_layers"], cfg.Dmax, cand, ws, mask=mask)
            T.talon_tree_attention(sl.q[:, :Np], sl.kp, sl.vp, sl.kt[:, :Np], sl.vt[:, :Np], mask, st.n_nodes, plen,
                                   cfg.L, out, None, wa)

        n, depth, rows, acc = [], [], [], []
        graphs = []
        for sl, tg in zip(slots, targets):
            step(sl)
            T.talon_target_argmax(tg, st, tgt, prob, sstat, vws)
            T.talon_greedy_accept(st, tgt, sstat, path, alen, bonus)
            torch.cuda.synchronize()
            n.append(int(st.n_nodes[0])); depth.append(int(st.depth_cur[0]))
            rows.append(int(st.n_nodes[0]) - int(st.frontier_count[0])); acc.append(int(alen[0]))
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                step(sl)
            graphs.append(g)
        for g in graphs:
            g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            graphs[i % n_slots].replay()
        torch.cuda.synchronize()
        us = (time.perf_counter() - t0) * 1e6 / steps
        rows_out.append({"N": v["N"], "mu": v["mu"], "init_layers": v["init_layers"], "us_per_step": us,
                         "steps_per_s": 1e6 / us, "n_mean": float(np.mean(n)), "depth_mean": float(np.mean(depth)),
                         "rows_scanned_mean": float(np.mean(rows)), "accepted_mean": float(np.mean(acc)),
                         "tau": float(np.mean(acc)) + 1.0})
        del graphs
    return rows_out


def literal_timing(T, torch, np, H, cfg, steps, n_slots):
    """Expansion alone, two ways on the same rotating inputs, each replayed as one HIP graph per
    slot: the capped single launch (per-row cap = the configuration's K) and the uncapped pool of
    Alg. 2 as written (one scan, plan, collect and select launch per layer).  Reports time per
    tree batch, tree sizes, depths, the largest fan-out and in how many sequences the trees differ."""
    slots = [Slot(cfg, cfg.seed + 1000 * i, torch, H) for i in range(n_slots)]
    dt = T.TALON_DTYPE_F32 if cfg.logits_dtype == "f32" else T.TALON_DTYPE_BF16
    roots = torch.from_numpy(H.root_tokens(cfg)).cuda()
    res = {"workload": cfg.name, "slots": n_slots, "steps": steps}
    trees = {}
    for mode in ("capped", "uncapped"):
        st = T.TreeState(cfg.B, cfg.N)
        mask = torch.zeros(cfg.B, st.N_pad, st.N_pad // 64, dtype=torch.int64, device="cuda")
        if mode == "capped":
            cand = T.Candidates(cfg.B, st.N_pad, cfg.K)
            ws = T.make_expand_workspace(cfg.B, st.N_pad, cfg.V, cfg.K, dt)

            def run(sl):
                T.talon_build_tree(roots, sl.logits, st, cfg.K, cfg.mu, cfg.K, 1, cfg.Dmax, cand, ws, mask=mask)
        else:
            ws = T.make_literal_workspace(cfg.B, st.N_pad, cfg.V, dt)

            def run(sl):
                T.talon_tree_init(st, roots)
                T.talon_expand_literal(sl.logits, st, cfg.Dmax, cfg.mu, cfg.K, 1, cfg.Dmax, ws)
                T.talon_build_tree_mask(st, mask)
        graphs, snap = [], []
        for sl in slots:
            run(sl)
            torch.cuda.synchronize()
            n = st.n_nodes.cpu().numpy()
            par = st.parent.cpu().numpy()
            snap.append((n.copy(), par.copy(), st.token.cpu().numpy().copy(), st.depth_cur.cpu().numpy().copy()))
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                run(sl)
            graphs.append(g)
        for g in graphs:
            g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            graphs[i % n_slots].replay()
        torch.cuda.synchronize()
        us = (time.perf_counter() - t0) * 1e6 / steps
        fan = max(int(np.bincount(par[b, 1:int(n[b])], minlength=1).max()) if n[b] > 1 else 0
                  for n, par, _, _ in snap for b in range(cfg.B))
        trees[mode] = snap
        res[mode] = {"us_per_call": us, "n_mean": float(np.mean([n.mean() for n, _, _, _ in snap])),
                     "layers_mean": float(np.mean([d.mean() for _, _, _, d in snap])), "largest_fan_out": fan}
    differ = 0
    for (n0, p0, t0_, _), (n1, p1, t1_, _) in zip(trees["capped"], trees["uncapped"]):
        for b in range(cfg.B):
            same = n0[b] == n1[b] and np.array_equal(p0[b, :n0[b]], p1[b, :n1[b]]) and np.array_equal(t0_[b, :n0[b]], t1_[b, :n1[b]])
            differ += 0 if same else 1
    res["sequences"] = n_slots * cfg.B
    res["sequences_whose_trees_differ"] = differ
    return res


def zipf_grid(T, torch, np, H, K=10, N=60, warm=20, runs=100):
    """Single-layer expansion latency on Zipf rows (the shape of the paper's App. E.6
    micro-benchmark): a tree of root + K children; the timed call expands those K parents by one
    layer (vocabulary scan of K rows + selection, one fused launch), once with the confidence
    gate of Alg. 2 and once with Alg. 1's top-K of the K x K pool.  HIP events around the
    launch (the library's hook); a long streaming-read launch is queued first so that the host
    is ahead of the device and the bracket holds device time only."""
    from workloads import WorkloadConfig, logits_row
    out = []
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    ballast = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").random_(0, 255)
    for V in (32000, 128256, 151936):
        for alpha in (0.7, 1.35, 5.0):
            cfg = WorkloadConfig(name="zipf", B=1, V=V, logits_dtype="bf16", K=K, N=N, Dmax=12, mu=0.03, Hq=8, Hkv=8,
                                 Dh=128, L=64, recipe=("zipf", alpha, 0.0))
            pool = np.zeros((1, cfg.N_pad, V), dtype=np.uint16)
            for i in range(K + 1):
                pool[0, i] = logits_row(cfg, cfg.seed, 0, i)
            dev = H.to_device_logits(pool)
            st = T.TreeState(1, N)
            cand = T.Candidates(1, st.N_pad, K)
            ws = T.make_expand_workspace(1, st.N_pad, V, K, T.TALON_DTYPE_BF16)
            roots = torch.from_numpy(H.root_tokens(cfg)).cuda()
            res = {"V": V, "alpha": alpha, "parents": K}
            for label, init_layers in (("adaptive_gate_us", 1), ("static_topk_us", 2)):
                us = []
                for it in range(warm + runs):
                    T.talon_probe_read(ballast, sink)
                    T.talon_tree_init(st, roots)
                    T.talon_expand_select_layer(dev, st, K, cfg.mu, K, init_layers, 12, cand, ws, layer=0)
                    T.talon_profile_scan_launches(True)
                    T.talon_expand_select_layer(dev, st, K, cfg.mu, K, init_layers, 12, cand, ws, layer=1)
                    torch.cuda.synchronize()
                    d, n_rec = T.talon_profile_read(1)
                    T.talon_profile_scan_launches(False)
                    assert n_rec == 1
                    if it >= warm:
                        us.append(d[0])
                res[label] = float(np.mean(us))
                res[label.replace("_us", "_new_nodes")] = int(st.n_nodes[0].item()) - 1 - K
            out.append(res)
    return out


def probes(T, torch):
    """Cycle counts (shader clock) of the two attention-step probes of the library."""
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    out = {"issue": [], "tile_loads": []}
    mixes = [(0, "32 exp2", 32), (1, "32 fma", 32), (2, "16 mfma 32x32x16 bf16, 4 accumulators", 16),
             (3, "16 mfma 32x32x16 bf16, 1 accumulator", 16), (4, "16 mfma + 32 (fma, exp2)", 16)]
    iters = 2000
    for waves in (4, 8):
        for mode, what, per_round in mixes:
            cyc = torch.zeros(8, dtype=torch.int64, device="cuda")
            T.talon_probe_issue(mode, waves, iters, cyc, sink)
            torch.cuda.synchronize()
            c = cyc.cpu().numpy()[:waves].astype(float) / iters
            out["issue"].append({"mix": what, "waves_per_simd": waves // 4, "cycles_per_round_first_wave": float(c[0]),
                                 "cycles_per_round_slowest_wave": float(c.max()),
                                 "cycles_per_instruction_slowest_wave": float(c.max()) / per_round})
    window = torch.zeros(16 << 20, dtype=torch.uint8, device="cuda")
    for waves in (4, 8):
        for loads in (4, 8):
            for with_mfma in (False, True):
                cyc = torch.zeros(2048, dtype=torch.int64, device="cuda")
                T.talon_probe_tile_loads(window, loads, with_mfma, waves, iters, cyc, sink)
                torch.cuda.synchronize()
                c = cyc.cpu().numpy().reshape(256, 8)[:, :waves].astype(float) / iters
                kb = waves * loads            # KB per compute unit and round
                out["tile_loads"].append({"waves": waves, "loads_per_wave": loads, "with_16_mfma": with_mfma,
                                          "KB_per_cu_round": kb, "cycles_per_round_mean": float(c.mean()),
                                          "cycles_per_round_slowest_wave": float(c.max()),
                                          "bytes_per_cycle_per_cu": kb * 1024.0 / float(c.mean())})
    return out


def attainable(T, torch):
    """Rates a plain kernel reaches on this device: read GB/s of a streaming pass over a buffer
    that no cache holds (three 1 GiB buffers in rotation, then 512 MiB pieces of them), and
    TFLOP/s of a register-resident bf16 MFMA loop on every SIMD (8 wavefronts per SIMD)."""
    bufs = [torch.empty(1 << 30, dtype=torch.uint8, device="cuda").random_(0, 255) for _ in range(3)]
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    out = {}
    for label, nbytes in (("read_1GiB", 1 << 30), ("read_512MiB", 1 << 29)):
        evs = []
        for i in range(12):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(); T.talon_probe_read(bufs[i % 3][:nbytes], sink); e1.record()
            evs.append((e0, e1))
        torch.cuda.synchronize()
        ms = sorted(e0.elapsed_time(e1) for e0, e1 in evs[3:])
        out[label] = {"us_median": ms[len(ms) // 2] * 1e3, "GBps": nbytes / (ms[len(ms) // 2] * 1e-3) / 1e9}
    wgs, iters = 256 * 8, 20000
    evs = []
    for i in range(6):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(); fl = T.talon_probe_mfma(wgs, iters, sink); e1.record()
        evs.append((e0, e1))
    torch.cuda.synchronize()
    ms = sorted(e0.elapsed_time(e1) for e0, e1 in evs[1:])
    out["mfma_bf16_32x32x16"] = {"us_median": ms[len(ms) // 2] * 1e3, "TFLOPs": fl / (ms[len(ms) // 2] * 1e-3) / 1e12}
    return out


def layerwise(T, torch, np, cfg, slots, st, cand, ws, roots, steps, elem):
    """Per-layer figures of the vocabulary scan: one fused launch per layer, HIP events around
    each (the library's measurement hook).  Rows come from an untimed pass that reads the
    frontier after every layer."""
    depth = min(cfg.Dmax, cfg.N - 1)
    n_slots = len(slots)
    rows = np.zeros((n_slots, depth))
    for i, s in enumerate(slots):
        T.talon_tree_init(st, roots)
        for d in range(depth):
            torch.cuda.synchronize()
            live = (st.status.cpu().numpy() & 11) == 0
            rows[i, d] = float((st.frontier_count.cpu().numpy() * live).sum())
            T.talon_expand_select_layer(s.logits, st, cfg.K, cfg.mu, cfg.K, 1, cfg.Dmax, cand, ws, layer=d)
    torch.cuda.synchronize()
    T.talon_profile_scan_launches(True)
    for i in range(steps):
        s = slots[i % n_slots]
        T.talon_tree_init(st, roots)
        for d in range(depth):
            T.talon_expand_select_layer(s.logits, st, cfg.K, cfg.mu, cfg.K, 1, cfg.Dmax, cand, ws, layer=d)
    torch.cuda.synchronize()
    us, n_rec = T.talon_profile_read(steps * depth)
    T.talon_profile_scan_launches(False)
    assert n_rec == steps * depth, (n_rec, steps, depth)
    us = np.asarray(us).reshape(steps, depth).mean(0)
    mean_rows = np.mean([rows[i % n_slots] for i in range(steps)], axis=0)
    out = []
    for d in range(depth):
        by = mean_rows[d] * cfg.V * elem
        out.append({"layer": d, "rows": round(float(mean_rows[d]), 2), "us": round(float(us[d]), 2),
                    "GBps": round(by / (us[d] * 1e-6) / 1e9, 1)})
    return out


def read_traffic(workload):
    """HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE + WRITE_SIZE, scaled by a
    copy kernel of known size); the summary under profiles/ holds `kernel: bytes` lines."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic_%s.txt" % workload)
    out = {}
    if os.path.exists(path):
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch "):
                _, kern, val = line.split()
                out[kern] = float(val)
    return out


def _oracle_steps(job):
    """Worker: whole oracle steps (Alg. 2 tree, mask, tree attention over all nodes and heads) of
    one configuration on fresh seeded inputs, one thread; input generation is not timed.
    Returns (steps done, seconds spent in the oracle)."""
    cfg_name, first_seed, budget_s, max_steps = job
    from threadpoolctl import threadpool_limits
    from oracle import talon_oracle as O
    from workloads import CONFIGS, attention_inputs, bf16_bits_to_f64, build_pool, root_tokens, storage_to_f64
    cfg = next(c for c in CONFIGS.values() if c.name == cfg_name)
    import numpy as np
    mu = float(np.float32(cfg.mu))
    n_done, busy = 0, 0.0
    with threadpool_limits(limits=1):
        while n_done < max_steps and busy < budget_s:
            seeds = [first_seed + 1000 * n_done] * cfg.B
            pool = build_pool(cfg, seeds)
            attn = [attention_inputs(cfg, seeds[b], b) for b in range(cfg.B)]
            roots = root_tokens(cfg)
            t0 = time.perf_counter()
            for b in range(cfg.B):
                rows = {}

                def row_of(i, b=b, rows=rows):
                    if i not in rows:
                        rows[i] = storage_to_f64(pool[b, i])
                    return rows[i]

                t = O.build_tree(row_of, int(roots[b]), N=cfg.N, K=cfg.K, mu=mu, cap=cfg.K, Dmax=cfg.Dmax, init_layers=1)
                m = O.build_tree_mask(t.parent)
                x, n = attn[b], t.n
                O.tree_attention(bf16_bits_to_f64(x["q"][:n]), bf16_bits_to_f64(x["k_prefix"]),
                                 bf16_bits_to_f64(x["v_prefix"]), bf16_bits_to_f64(x["k_tree"][:n]),
                                 bf16_bits_to_f64(x["v_tree"][:n]), m)
            busy += time.perf_counter() - t0
            n_done += 1
    return n_done, busy


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(cfg, budget_s):
    """The CPU oracle, as it stands, timed on this host on whole steps of the same workload:
    one thread, then one single-threaded worker process per core (independent steps side by
    side: the whole-job rate of the host).  Must run before this process initialises the GPU."""
    import multiprocessing as mp
    nproc = os.cpu_count() or 1
    try:
        usable = len(os.sched_getaffinity(0))
    except AttributeError:
        usable = nproc
    cores = max(1, min(usable, 16))     # one GPU's share of the host
    one_n, one_busy = _oracle_steps((cfg.name, cfg.seed, budget_s / 2.0, 50))
    with mp.get_context("fork").Pool(cores) as pool:
        res = pool.map(_oracle_steps, [(cfg.name, cfg.seed + 100000 * (w + 1), budget_s / 2.0, 50) for w in range(cores)])
    rate_all = sum(n / busy for n, busy in res)
    return {"value": rate_all, "unit": "steps/s", "cores": cores, "kind": "oracle",
            "single_thread_value": one_n / one_busy, "nproc": nproc, "cpu_model": cpu_model(),
            "sample": "%d whole steps of %s on one thread, then %d steps on %d single-threaded worker processes side by "
                      "side (expansion + mask + attention over all nodes and heads; numpy fp64, BLAS pinned to one "
                      "thread per process; input generation not timed)" % (one_n, cfg.name, sum(n for n, _ in res), cores)}


if __name__ == "__main__":
    main()
