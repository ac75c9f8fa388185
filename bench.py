#!/usr/bin/env python3
"""Benchmark of the DySpec verification hot path on one MI355X.

One step = one pass of the whole path over one batch of synthetic input: tree attention for
every layer of the model shape (dyspec_tree_attn, L launches) followed by the vocabulary
softmax + tree rejection sampling (dyspec_verify).  The token tree is built once, before
the timed region, by dyspec_build_tree from the same draft logits.  Every input is already
resident in HBM when timing starts.

Prints ONE JSON line: verified tree tokens/s, the roofline position of the dominant kernel
(the matrix-core tree-attention kernel) and the CPU oracle timed on a bounded sample.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "verified tree tokens/s (tree-attn + verify), 70B shape, 1 GPU; % of HBM peak"
PEAK_BF16_TFLOPS = 2500.0        # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0            # MI355X HBM3E


def measured_traffic(workload: str):
    """HBM bytes per tree-attention launch from the two rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE, each
    scaled by what the same counter reads for a 1 GiB device copy) summarised under profiles/, and the commit
    they were measured at: one line per workload in profiles/hbm_traffic_per_launch.txt, rewritten whenever
    the profiles are regenerated.  (None, None) for a workload that was not profiled."""
    try:
        with open(os.path.join(ROOT, "profiles", "hbm_traffic_per_launch.txt")) as f:
            for line in f:
                parts = line.split()
                if len(parts) >= 3 and not line.startswith("#") and parts[0] == workload:
                    return int(parts[1]), parts[2]
    except OSError:
        pass
    return None, None


def tree_only_sweep(dy, synth, torch, np, dev) -> int:
    """Block-sparsity friendly token order (the paper's appendix on token order and its random-tree table):
    tree attention alone, 64 heads x head_dim 128, no prefix, on trees in creation order and after
    dyspec_dfs_reorder; also the number of non-empty 32x32 blocks of the ancestor mask either way."""
    H, d, scale = 64, 128, 1.0 / math.sqrt(128)

    def blocks(mask_i64, n):
        m = mask_i64.cpu().numpy().view(np.uint64)
        bits = ((m[:n, :, None] >> np.arange(64, dtype=np.uint64)[None, None, :]) & np.uint64(1)).astype(bool)
        dense = np.zeros((-(-n // 32) * 32,) * 2, dtype=bool)
        dense[:n, :n] = bits.reshape(n, -1)[:, :n]
        return int(dense.reshape(dense.shape[0] // 32, 32, -1, 32).any(axis=(1, 3)).sum())

    def time_attn(q, kt, vt, mask, batch, reps=40):
        empty = torch.empty((0, H, d), dtype=q.dtype, device=dev)
        out = torch.empty_like(q)
        for _ in range(5):
            dy.tree_attn(q, empty, empty, kt, vt, mask, batch, scale, out=out)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        best = float("inf")
        for _ in range(3):                 # best of three runs of `reps` launches
            torch.cuda.synchronize()
            e0.record()
            for _ in range(reps):
                dy.tree_attn(q, empty, empty, kt, vt, mask, batch, scale, out=out)
            e1.record()
            torch.cuda.synchronize()
            best = min(best, e0.elapsed_time(e1) * 1e3 / reps)
        return best

    rows = []
    for n in (256, 512, 1024, 2048):
        batch = dy.Batch.from_sizes([n], [0])
        g = torch.Generator(device=dev).manual_seed(n)
        q, kt, vt = (torch.randn((n, H, d), generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16) for _ in range(3))
        for kind in ("random", "greedy") if n <= dy.MAX_BUILD_NODES else ("random",):    # the builder stops at 1024 rows
            if kind == "random":           # parent of node i uniform among the earlier nodes, children in index order
                rng = np.random.default_rng(n)
                par = np.full(n, -1, np.int32)
                par[1:] = [rng.integers(0, i) for i in range(1, n)]
                fc, ns, last = np.full(n, -1, np.int32), np.full(n, -1, np.int32), np.full(n, -1, np.int32)
                dep, rk, cnt = np.zeros(n, np.int32), np.zeros(n, np.int32), np.zeros(n, np.int32)
                for i in range(1, n):
                    p = par[i]
                    dep[i], rk[i] = dep[p] + 1, cnt[p]
                    cnt[p] += 1
                    if last[p] < 0:
                        fc[p] = i
                    else:
                        ns[last[p]] = i
                    last[p] = i
                mk = lambda a: torch.from_numpy(a).to(dev)
                tree = dy.Tree(mk(par), mk(np.zeros(n, np.int32)), mk(rk), mk(fc), mk(ns), mk(dep))
                m = np.zeros((n, batch.mask_words), np.uint64)
                for j in range(n):
                    a = j
                    while a >= 0:
                        m[j, a // 64] |= np.uint64(1) << np.uint64(a % 64)
                        a = par[a]
                mask = torch.from_numpy(m.view(np.int64)).to(dev)
            else:                          # the builder's own tree on N(0, 3^2) logits at temperature 0.6
                cfg = synth.CONFIGS["llama2_70b"]
                rng = np.random.default_rng(7 * n)
                logits = torch.from_numpy((rng.standard_normal((n, cfg.vocab)) * 3.0).astype(np.float32)).to(dev)
                built = dy.build_tree(logits, batch, (0.6,), 3)
                tree, mask = built.tree, built.anc_mask
            re = dy.dfs_reorder(tree, batch)
            idx = re.gather_index(batch)
            t0 = time_attn(q, kt, vt, mask, batch)
            t1 = time_attn(q[idx].contiguous(), kt[idx].contiguous(), vt[idx].contiguous(), re.anc_mask, batch)
            rows.append({"tree": kind, "nodes": n, "blocks_creation_order": blocks(mask, n), "blocks_dfs_order": blocks(re.anc_mask, n),
                         "us_creation_order": round(t0, 2), "us_dfs_order": round(t1, 2),
                         "max_depth": int(tree.depth.max().item())})
    print(json.dumps({"tree_only_sweep": {"heads": H, "head_dim": d, "block": 32, "dtype": "bf16", "rows": rows}}))
    return 0


def tree_builders(dy, synth, torch, np, dev, cfg) -> int:
    """The two tree builders on the workload's draft table (outside the metric): the greedy fixed-budget
    builder (Algorithm 1, N - 1 dependent draws in one workgroup per sequence) and the threshold builder
    (Algorithm 2, every node of a level in its own workgroup), the latter at the smallest value the greedy
    run opened and with 1.5 x the rows, as the paper relaxes the budget.  Wall time of the calls, synchronised."""
    draft_h, _ = synth.make_logits(cfg)
    cap = [min(n + n // 2, 1024) for n in cfg.n_nodes]
    # rows past a sequence's own N repeat its first rows: the table only has to be large enough
    parts, off = [], 0
    for n, c in zip(cfg.n_nodes, cap):
        rows = draft_h[off:off + n]
        parts.append(np.concatenate([rows, rows[:c - n]]) if c > n else rows)
        off += n
    wide = torch.from_numpy(np.concatenate(parts)).to(dev)
    draft = torch.from_numpy(draft_h).to(dev)
    b_greedy, b_thr = dy.Batch.from_sizes(cfg.n_nodes), dy.Batch.from_sizes(cap)

    def wall(fn, reps=3):
        best, out = float("inf"), None
        for _ in range(reps):
            torch.cuda.synchronize()
            t = time.perf_counter()
            out = fn()
            torch.cuda.synchronize()
            best = min(best, time.perf_counter() - t)
        return best * 1e3, out

    ms_g, greedy = wall(lambda: dy.build_tree(draft, b_greedy, cfg.temps, cfg.seed))
    est = greedy.est_value.cpu().numpy().astype(np.float64)
    nb = greedy.n_built.cpu().numpy()
    thr, off = [], 0
    for n, k in zip(cfg.n_nodes, nb):
        thr.append(float(est[off:off + k].min()))
        off += n
    ms_t, (built, levels) = wall(lambda: dy.build_tree_threshold(wide, b_thr, cfg.temps, thr, cfg.seed))
    line = {"mode": "tree-builders", "workload": cfg.name, "vocab": cfg.vocab,
            "greedy": {"rows": [int(x) for x in nb], "ms": round(ms_g, 3)},
            "threshold": {"t": [round(x, 6) for x in thr], "capacity": cap,
                          "rows": [int(x) for x in built.n_built.cpu().numpy()], "levels": levels, "ms": round(ms_t, 3)}}
    print(json.dumps(line))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="llama2_70b")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="target CPU time of the oracle sample")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also launch one plain 1 GiB device copy (a known-size reference for HBM byte counters)")
    ap.add_argument("--tree-only-sweep", action="store_true",
                    help="instead of the step benchmark: tree-only attention (64 heads, head_dim 128, no prefix) on random "
                         "and greedy trees of 256..2048 nodes, creation order against depth-first order")
    ap.add_argument("--target-temp", type=float, default=None,
                    help="target temperature of every sequence in verification (0 = the paper's temperature-0 "
                         "target); default: the workload's own temperatures, as for the draft")
    ap.add_argument("--batched-layers", action="store_true",
                    help="attention of all layers through ONE dyspec_tree_attn_layers call per step instead of one "
                         "dyspec_tree_attn call per layer (same work; not what a model whose layers depend on each "
                         "other can do, so the default and the headline value stay per layer)")
    ap.add_argument("--tree-builders", action="store_true",
                    help="instead of the step benchmark: time the greedy and the threshold tree builder on the workload's draft table")
    ap.add_argument("--bf16-logits", action="store_true",
                    help="verification reads bf16 logit tables (dyspec_verify_bf16): the fp32 tables rounded once, "
                         "half the bytes of the statistics pass; the tree is built from the same rounded values")
    ap.add_argument("--dfs-order", action="store_true",
                    help="rename the tree's nodes in depth-first order (dyspec_dfs_reorder) before attention and "
                         "verification: subtrees become runs of rows, fewer tree tiles per workgroup")
    ap.add_argument("--no-ceilings", action="store_true",
                    help="skip the two measured ceilings (MFMA-only loop, streaming HBM read)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding or collectives); use --gpus 1",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2410_11744_amd as dy
    from paper_2410_11744_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    dy.load_library()
    dy.init()                          # code loading and kernel attributes now, not inside the first steps
    dev = torch.device("cuda:0")
    if args.tree_only_sweep:
        return tree_only_sweep(dy, synth, torch, np, dev)
    cfg = synth.CONFIGS[args.workload]
    if args.tree_builders:
        return tree_builders(dy, synth, torch, np, dev, cfg)
    target_temps = cfg.temps if args.target_temp is None else (args.target_temp,) * len(cfg.n_nodes)
    batch = dy.Batch.from_sizes(cfg.n_nodes, cfg.prefix_len)
    n_tokens = batch.total_nodes
    scale = 1.0 / math.sqrt(cfg.head_dim)

    # ---- inputs (resident in HBM before timing)
    draft_h, target_h = synth.make_logits(cfg)
    if args.bf16_logits:               # every consumer (builder, verification, oracle) sees the rounded values
        draft_h = torch.from_numpy(draft_h).to(torch.bfloat16).float().numpy()
        target_h = torch.from_numpy(target_h).to(torch.bfloat16).float().numpy()
    draft, target = torch.from_numpy(draft_h).to(dev), torch.from_numpy(target_h).to(dev)
    built = dy.build_tree(draft, batch, cfg.temps, cfg.seed)
    # the builder is outside the timed region (the metric names tree attention + verification);
    # its time is reported next to it: the second call, HIP events around the library call
    eb = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    torch.cuda.synchronize()
    eb[0].record()
    dy.build_tree(draft, batch, cfg.temps, cfg.seed)
    eb[1].record()
    torch.cuda.synchronize()
    build_tree_ms = eb[0].elapsed_time(eb[1])
    if args.dfs_order:
        # the paper's token order for attention (Appendix C): nodes renamed in depth-first order, the
        # rows of the logit tables follow their nodes; verification does not depend on the numbering
        re = dy.dfs_reorder(built.tree, batch)
        idx = re.gather_index(batch)
        draft, target = draft[idx].contiguous(), target[idx].contiguous()
        idx_h = idx.cpu().numpy()
        draft_h, target_h = draft_h[idx_h], target_h[idx_h]
        built = dy.BuiltTrees(re.tree, built.est_value[idx].contiguous(), re.anc_mask, built.n_built)
    v_draft, v_target = (draft.to(torch.bfloat16), target.to(torch.bfloat16)) if args.bf16_logits else (draft, target)
    # all layers' tensors live in five stacked allocations [L, ...]; the per-layer calls take views
    stacked = None
    for l in range(cfg.layers):
        one = synth.make_attention_inputs(cfg, l, device=dev)
        if stacked is None:
            stacked = [torch.empty((cfg.layers,) + tuple(t.shape), dtype=t.dtype, device=dev) for t in one]
        for k in range(5):
            stacked[k][l].copy_(one[k])
        del one
    layers = [tuple(t[l] for t in stacked) for l in range(cfg.layers)]
    out_stack = torch.empty_like(stacked[0])
    outs = [out_stack[l] for l in range(cfg.layers)]
    vout = dy.VerifyOutput.empty(batch, dev)
    torch.cuda.synchronize()
    depth = built.tree.depth.cpu().numpy().astype(np.int64)
    n_built = built.n_built.cpu().numpy()

    # the step's calls, arguments checked and marshalled once as a decode loop would: at the short
    # shapes a layer's kernel runs for less time than the binding's per-call checks take on the host
    layer_calls = [dy.tree_attn_call(*layers[l], built.anc_mask, batch, scale, out=outs[l]) for l in range(cfg.layers)]
    verify_step = dy.verify_call(v_draft, v_target, batch, built.tree, cfg.temps, target_temps, cfg.seed, out=vout)

    def step(ev=None):
        if ev:
            ev[0].record()
        if args.batched_layers:
            dy.tree_attn_layers(*stacked, built.anc_mask, batch, scale, out=out_stack)
        else:
            for call in layer_calls:
                call()
        if ev:
            ev[1].record()
        verify_step()
        if ev:
            ev[2].record()

    if args.copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)                       # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst
    # ---- measured ceilings of this chip, beside the published peaks
    ceilings = None
    if not args.no_ceilings:
        sink = torch.zeros(1, dtype=torch.float32, device=dev)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        dy.probe_mfma_bf16(2000, sink)
        torch.cuda.synchronize()
        e0.record()
        fl = dy.probe_mfma_bf16(20000, sink)
        e1.record()
        torch.cuda.synchronize()
        mfma_tflops = fl / (e0.elapsed_time(e1) * 1e-3) / 1e12
        dy.probe_mfma_bf16(2000, sink, random_operands=True)
        torch.cuda.synchronize()
        e0.record()
        fl = dy.probe_mfma_bf16(20000, sink, random_operands=True)
        e1.record()
        torch.cuda.synchronize()
        mfma_random_tflops = fl / (e0.elapsed_time(e1) * 1e-3) / 1e12
        # a loop of nothing but MFMAs keeps the matrix pipe of every SIMD busy every cycle:
        # 1024 SIMDs x 32768 flops per 32 cycles, so the rate names the clock it ran at
        implied_ghz = lambda tf: tf * 1e12 / (1024 * 1024) / 1e9
        buf = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        best = float("inf")
        for _ in range(5):
            torch.cuda.synchronize()
            e0.record()
            nbytes = dy.probe_hbm_read(buf, sink)
            e1.record()
            torch.cuda.synchronize()
            best = min(best, e0.elapsed_time(e1))
        del buf
        ceilings = {"mfma_bf16_tflops": round(mfma_tflops, 1), "mfma_bf16_clock_ghz": round(implied_ghz(mfma_tflops), 3),
                    "mfma_bf16_random_operands_tflops": round(mfma_random_tflops, 1),
                    "mfma_bf16_random_operands_clock_ghz": round(implied_ghz(mfma_random_tflops), 3),
                    "hbm_read_gbs": round(nbytes / (best * 1e-3) / 1e9, 1),
                    "how": "MFMA: 8192 waves of independent 32x32x16 bf16 MFMAs, no memory or vector work, operands a smooth "
                           "ramp of small values or random in +-[0.25, 4); the clock is the one at which 1024 busy matrix "
                           "pipes give that rate (nominal 2.4 GHz); HBM: one streaming read of 1 GiB, best of 5"}

    # Untimed warmup.  The interpreter's own cyclic garbage collector is parked first: every binding
    # call creates a few ctypes objects, and once enough have piled up CPython runs a full collection
    # that walks every object torch and numpy hold -- 35-40 ms on the host inside whichever call
    # triggers it (measured with gc.callbacks: it is the one slow launch a process used to show around
    # its 350th dispatch; a plain HIP program launching the same kernels shows none).  What exists now
    # is moved to the permanent generation, as serving loops do; collection stays enabled.
    import gc
    gc.collect()
    gc.freeze()
    warmup = args.warmup
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(evs[k])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    attn_ms = sum(e[0].elapsed_time(e[1]) for e in evs) / args.steps
    verify_ms = sum(e[1].elapsed_time(e[2]) for e in evs) / args.steps
    value = n_tokens / (ms_per_step * 1e-3)

    # ---- the shader clock under this workload (after the timed region): one sleeping wave on a
    #      stream of its own counts shader cycles and wall-clock ticks while a few more steps run
    shader_clock_ghz = None
    if not args.no_ceilings:
        k2 = max(3, min(args.steps, int(60.0 / max(ms_per_step, 1e-3))))       # about 60 ms of steps
        naps = int(max(1, min(1 << 24, 0.4 * k2 * ms_per_step * 1e-3 * 2.4e9 / 8128)))
        counters = torch.zeros(2, dtype=torch.int64, device=dev)
        side = torch.cuda.Stream()
        torch.cuda.synchronize()
        step()
        with torch.cuda.stream(side):
            khz = dy.probe_clock(naps, counters)
        for _ in range(k2 - 1):
            step()
        torch.cuda.synchronize()
        cyc, ticks = (int(x) for x in counters.cpu().numpy())
        if ticks > 0:
            shader_clock_ghz = round(cyc / (ticks / (khz * 1e3)) / 1e9, 3)

    # ---- roofline of the dominant kernel (tree attention, one launch = one layer)
    # Algorithmic work per launch: every row scores and accumulates over all prefix keys and
    # over its ancestors-or-self in the tree: 4*d flops per (row, visible key).
    visible = sum(int(cfg.prefix_len[s]) * int(cfg.n_nodes[s]) for s in range(batch.n_seq)) + int((depth + 1).sum())
    flops_per_launch = 4.0 * cfg.n_q_heads * cfg.head_dim * visible
    launch_ms = attn_ms / cfg.layers
    achieved_tflops = flops_per_launch / (launch_ms * 1e-3) / 1e12
    elt = 4 if cfg.dtype == "f32" else 2
    bytes_attn_launch = elt * cfg.head_dim * (2 * cfg.n_kv_heads * (batch.total_prefix + n_tokens)
                                              + 2 * cfg.n_q_heads * n_tokens)
    bytes_step = bytes_attn_launch * cfg.layers + (4.0 if args.bf16_logits else 8.0) * n_tokens * cfg.vocab
    hbm_gbs = bytes_step / (ms_per_step * 1e-3) / 1e9
    # which roof bounds the kernel at this shape: flops per algorithmic byte against the ridge
    ridge = PEAK_BF16_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9)
    kernel = "tree_attn_mfma_kernel<%d, 1>" % cfg.head_dim if cfg.dtype == "bf16" else "tree_attn_simple_kernel<float, %d>" % ((cfg.head_dim // 4 + 15) // 16)
    if cfg.dtype == "bf16" and flops_per_launch / bytes_attn_launch >= ridge:
        roofline = {"kernel": kernel, "bound": "mfma", "achieved": round(achieved_tflops, 2), "peak": PEAK_BF16_TFLOPS,
                    "unit": "TFLOP/s", "frac": round(achieved_tflops / PEAK_BF16_TFLOPS, 4)}
        if ceilings:
            roofline["frac_of_measured_ceiling"] = round(achieved_tflops / ceilings["mfma_bf16_tflops"], 4)
    else:
        gbs = bytes_attn_launch / (launch_ms * 1e-3) / 1e9
        roofline = {"kernel": kernel, "bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS,
                    "unit": "GB/s", "frac": round(gbs / PEAK_HBM_GBS, 4)}
        if ceilings:
            roofline["frac_of_measured_ceiling"] = round(gbs / ceilings["hbm_read_gbs"], 4)
    if args.batched_layers:        # one launch covers all layers: figures below stay per layer (time / layers)
        roofline["note"] = f"one launch for {cfg.layers} layers; launch_us, flops and bytes are per layer"
    traffic, traffic_commit = (None, None) if args.batched_layers else measured_traffic(args.workload)
    roofline.update({"traffic": traffic, "traffic_measured_at_commit": traffic_commit,
                     "launch_us": round(launch_ms * 1e3, 2),
                     "flops_per_launch": flops_per_launch, "algorithmic_bytes_per_launch": bytes_attn_launch,
                     "achieved_tflops": round(achieved_tflops, 2)})

    # ---- CPU oracle on a bounded sample of the same workload (reported baseline, not a target)
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        q, kp, vp, kt, vt = [t.float().cpu().numpy() for t in layers[0]]
        mask = built.anc_mask.cpu().numpy().view(np.uint64)
        rng = np.random.default_rng(0)
        total_rows = n_tokens * cfg.n_q_heads
        N0, P0 = int(cfg.n_nodes[0]), int(cfg.prefix_len[0])      # sample rows from sequence 0
        words0 = (N0 + 63) // 64
        m0 = np.ascontiguousarray(mask[:N0, :words0])

        def run(n_rows):
            pick = rng.choice(N0 * cfg.n_q_heads, n_rows, replace=False)
            rj, rh = np.divmod(pick, cfg.n_q_heads)
            t = time.perf_counter()
            oracle.tree_attn_rows(q[:N0], kp[:P0], vp[:P0], kt[:N0], vt[:N0], m0, scale, rj, rh)
            return time.perf_counter() - t
        t_probe = run(256)
        # all (row, head) pairs of sequence 0 in layer 0, repeated (fresh row order each time) until
        # the sample has used about --cpu-seconds of wall time
        per_pass = int(min(N0 * cfg.n_q_heads, max(256, 256 * args.cpu_seconds / max(t_probe, 1e-4))))
        n_rows, t_rows = 0, 0.0
        while t_rows < args.cpu_seconds and n_rows < 64 * per_pass:
            t_rows += run(per_pass)
            n_rows += per_pass
        # rows of sequence 0 see P0 + ancestors keys; scale to the whole batch by visible keys
        vis0 = P0 * N0 + int((depth[:N0] + 1).sum())
        t_attn_step = t_rows / n_rows * (N0 * cfg.n_q_heads) * (visible / vis0) * cfg.layers
        t = time.perf_counter()
        off = 0
        for s, n in enumerate(cfg.n_nodes):
            tr = {k: getattr(built.tree, k).cpu().numpy()[off:off + n] for k in ("token", "first_child", "next_sibling")}
            oracle.verify(draft_h[off:off + n], target_h[off:off + n], tr["token"], tr["first_child"],
                          tr["next_sibling"], float(np.float32(cfg.temps[s])), float(np.float32(target_temps[s])),
                          cfg.seed, seq=s)
            off += n
        t_verify = time.perf_counter() - t
        # the same oracle on one thread, on a sample a tenth as long (figure beside the all-threads one)
        all_threads = oracle.num_threads()
        oracle.set_num_threads(1)
        rows_1 = max(64, int(per_pass * max(args.cpu_seconds, 1.0) * 0.1 / max(t_rows / max(n_rows, 1) * per_pass * all_threads, 1e-6)))
        rows_1 = min(rows_1, N0 * cfg.n_q_heads)
        t_1 = run(rows_1)
        oracle.set_num_threads(all_threads)
        t_attn_step_1 = t_1 / rows_1 * (N0 * cfg.n_q_heads) * (visible / vis0) * cfg.layers
        cpu = {"value": round(n_tokens / (t_attn_step + t_verify), 3), "unit": "tokens/s",
               "cores": all_threads, "kind": "oracle",
               "one_thread_value": round(n_tokens / (t_attn_step_1 + t_verify), 4),
               "one_thread_sample": f"{rows_1} row evaluations in {t_1:.2f} s on one thread, scaled the same way",
               "sample": f"tree attention: {n_rows} row evaluations on layer 0's tensors (of {total_rows * cfg.layers} "
                         f"(row, head, layer) rows per step) in {t_rows:.2f} s, scaled by row count; "
                         f"verification walk in full ({t_verify * 1e3:.1f} ms)"}

    line = {
        "metric": METRIC, "value": round(value, 1), "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype if cfg.dtype != "f32" else "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {cfg.layers} layers, {cfg.n_q_heads}q/{cfg.n_kv_heads}kv heads, "
                               f"head_dim {cfg.head_dim}, prefix {list(cfg.prefix_len)}, tree rows {list(cfg.n_nodes)}, "
                               f"vocab {cfg.vocab}, batch {batch.n_seq}",
                   "node_order": "depth-first (dyspec_dfs_reorder)" if args.dfs_order else "creation order",
                   "logit_tables": "bf16" if args.bf16_logits else "fp32",
                   "attention_call": "dyspec_tree_attn_layers, one call per step" if args.batched_layers
                                     else "dyspec_tree_attn, one call per layer",
                   "draft_temp": [float(x) for x in cfg.temps], "target_temp": [float(x) for x in target_temps],
                   "tree_rows_built": [int(x) for x in n_built], "max_depth": int(depth.max())},
        "attn_ms_per_step": round(attn_ms, 4), "verify_ms_per_step": round(verify_ms, 4),
        "n_accepted": [int(x) for x in vout.n_accepted.cpu().numpy()],
        "build_tree_ms_outside_the_step": round(build_tree_ms, 3),
        "pct_hbm_peak": round(100.0 * hbm_gbs / PEAK_HBM_GBS, 2), "algorithmic_gbs": round(hbm_gbs, 1),
        "shader_clock_ghz_under_this_workload": shader_clock_ghz,
        "roofline": roofline, "cpu_baseline": cpu, "ceilings": ceilings,
    }
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
