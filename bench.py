#!/usr/bin/env python3
"""Benchmark of the transit-parallel sampling path on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input:
one nd_sample call (transit enumeration, grouping by transit, scheduling
classes, the sampling kernels, output compaction) over every root of the
workload.  Inputs are resident in HBM before the timed region.  Prints one JSON
line.  Without --workload the line is for the largest k-hop workload (c5_khop)
and carries, under "also", the same measurements for the largest random-walk
workload (c5_deepwalk), both timed in this one run.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--mode tp|sp]
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

HBM_PEAK_GBS = 8000.0

# HBM bytes per launch of the dominant kernel from two rocprofv3 --pmc runs of this file
# (FETCH_SIZE, then WRITE_SIZE; scaled by the factors the copy kernel of `--workload copy_calib`
# gives: x2.0 and x1.0), averaged over the launches of one call.  Sources: the counter tables in
# profiles/c5_khop_tp_rocprofv3.md and profiles/c5_deepwalk_tp_rocprofv3.md.  None where not profiled.
MEASURED_TRAFFIC_BYTES = {
    ("c5_khop", "tp", "sample_sub"): 3162426811,        # 1,337.6 MiB fetched + 1,678.4 MiB written per launch
    ("c5_deepwalk", "tp", "walk_window"): 52888034690,  # 48,813.0 MiB fetched + 1,625.0 MiB written per launch
}

WORKLOADS = {
    # name: (graph builder, app, params, description)
    "c5_khop": ("config5_graph", "khop", dict(num_steps=2, fanout=[25, 10]),
                "k-hop [25,10], every vertex a root, R-MAT scale 22 (int64 offsets)"),
    "c5_khop_unique": ("config5_graph", "khop", dict(num_steps=2, fanout=[25, 10], unique_rounds=4),
                       "k-hop [25,10] with unique neighbours (4 rounds), every vertex a root, R-MAT scale 22"),
    "c5_deepwalk": ("config5_graph", "deepwalk", dict(num_steps=100),
                    "DeepWalk length 100, one walk per vertex, R-MAT scale 22"),
    "c3_khop": ("config3_graph", "khop", dict(num_steps=2, fanout=[25, 10]),
                "k-hop [25,10], every vertex a root (228 batches of 1,024 in one call), 233K dense"),
    "c4_khop": ("config4_graph", "khop", dict(num_steps=2, fanout=[25, 10]),
                "k-hop [25,10], every vertex a root, 3M power-law (468 MB of adjacency: beyond the last-level cache)"),
    "c2_node2vec": ("config2_graph", "node2vec", dict(num_steps=100, p=2.0, q=0.5, use_weights=1),
                    "node2vec p=2 q=0.5 length 100, 57K power-law, weights U[1,5)"),
    "c2_ppr": ("config2_graph", "ppr", dict(num_steps=100, term_prob=0.01, use_weights=1),
               "PPR termination 0.01 cap 100, 57K power-law, weights U[1,5)"),
    "c1_deepwalk": ("config1_graph", "deepwalk", dict(num_steps=100),
                    "DeepWalk length 100, R-MAT scale 12"),
    "c5_multirw": ("config5_graph", "multirw", dict(num_steps=100, roots_per_sample=100),
                   "multi-dimensional walk, 100 roots per sample, length 100, 41,943 samples, R-MAT scale 22"),
    "c4_layer": ("config4_graph", "layer", dict(num_steps=2, fanout=[2048, 2048], roots_per_sample=64),
                 "layer sampling 64 roots, 2 x 2,048, 4,096 batches, 3M power-law"),
    "c4_layer_symmetric": ("config4_graph", "layer",
                           dict(num_steps=2, fanout=[2048, 2048], roots_per_sample=64, use_weights=1),
                           "layer sampling over edge weights 2^14 / (deg(v) deg(u)) (symmetric normalisation), "
                           "64 roots, 2 x 2,048, 4,096 batches, 3M power-law"),
}


def bench_layer_edges(args, B, inputs, torch, np):
    """Layer sampling followed by the edges between consecutive layers (Section 4.2, importance
    sampling): per call one nd_sample and, for each of the two steps, nd_layer_edges_count, the
    8-byte read of the total, and nd_layer_edges_fill into a buffer of that size."""
    g = inputs.config4_graph()
    sys.stderr.write(f"[bench] {g.describe()}\n")
    dg = B.nd_graph_create(g.row_offsets, g.col_indices)
    nb, R, fan = 4096, 64, [2048, 2048]
    roots = torch.as_tensor(inputs.permutation(g.V, 4)[:nb * R].copy(), device="cuda:0")
    p = B.nd_params_init(num_steps=2, fanout=fan, roots_per_sample=R)
    s = B.Sampler(dg, B.ND_LAYER, p, nb * R)
    shapes = [(nb, R), (nb, fan[0]), (nb, fan[1])]
    ws = [torch.empty(B.nd_layer_edges_workspace_bytes(nb, shapes[i][1]), dtype=torch.uint8, device="cuda:0")
          for i in range(2)]
    row_ptr = [torch.empty(nb * shapes[i][1] + 1, dtype=torch.int64, device="cuda:0") for i in range(2)]
    ev = lambda: torch.cuda.Event(enable_timing=True)
    t_sample = t_count = t_fill = 0.0
    edges = [0, 0]
    e_all0, e_all1 = ev(), ev()
    for it in range(args.warmup + args.steps):
        if it == args.warmup:
            torch.cuda.synchronize()
            t_sample = t_count = t_fill = 0.0
            e_all0.record()
        e = [ev() for _ in range(6)]
        e[0].record()
        out = s.run(roots, 1)
        e[1].record()
        layers = [roots.view(nb, R), out[0].view(nb, fan[0]), out[1].view(nb, fan[1])]
        marks = []
        for i in range(2):
            a, b, c = ev(), ev(), ev()
            a.record()
            B.nd_layer_edges_count(dg, layers[i], layers[i + 1], row_ptr[i], ws[i])
            b.record()
            edges[i] = int(row_ptr[i][-1].item())
            slots = torch.empty(edges[i], dtype=torch.int32, device="cuda:0")
            b2 = ev()
            b2.record()
            B.nd_layer_edges_fill(dg, layers[i], layers[i + 1], row_ptr[i], slots)
            c.record()
            marks.append((a, b, b2, c))
        torch.cuda.synchronize()
        t_sample += e[0].elapsed_time(e[1])
        for a, b, b2, c in marks:
            t_count += a.elapsed_time(b)
            t_fill += b2.elapsed_time(c)
    e_all1.record()
    torch.cuda.synchronize()
    ms = e_all0.elapsed_time(e_all1) / args.steps
    k = args.steps
    # what a pass over every transit slot would stream (the adjacency lists of all transits), and what
    # each of the two passes does stream: the list of every distinct transit of a sample once
    deg = torch.as_tensor(np.diff(g.row_offsets).astype(np.int64), device="cuda:0")
    streamed = [int((deg[layers[i].reshape(-1).clamp(min=0).long()] * (layers[i].reshape(-1) >= 0)).sum().item())
                for i in range(2)]
    distinct = []
    for i in range(2):
        tot = 0
        for b0 in range(0, nb, 512):
            srt, _ = torch.sort(layers[i][b0:b0 + 512].long(), dim=1)
            first = torch.ones_like(srt, dtype=torch.bool)
            first[:, 1:] = srt[:, 1:] != srt[:, :-1]
            tot += int((deg[srt.clamp(min=0)] * (first & (srt >= 0))).sum().item())
        distinct.append(tot)
    print(json.dumps({
        "metric": "edges recorded/s (layer sampling + edges between consecutive layers)",
        "value": round(sum(edges) / (ms * 1e-3), 1), "unit": "edges/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms, 4), "higher_is_better": True, "dtype": "int32",
        "data": "synthetic",
        "config": {"workload": "c4_layer_edges", "graph": g.describe(), "samples": nb, "layers": [R] + fan,
                   "edges_per_step": edges, "adjacency_entries_of_all_transit_slots": streamed,
                   "adjacency_entries_streamed_per_pass": distinct},
        "phase_ms_per_step": {"sample": round(t_sample / k, 4), "edges_count": round(t_count / k, 4),
                              "edges_fill": round(t_fill / k, 4)},
        # the two counting passes of a call (edges_kernel + the row-pointer scan): 4 bytes per streamed
        # adjacency entry + 4 per transit slot and per new vertex read + 4 per transit slot written,
        # over their time between HIP events on the launch stream
        "roofline": _edges_roofline(distinct, shapes, nb, t_count / k)}))


def _edges_roofline(distinct, shapes, nb, count_ms):
    algorithmic = sum(4 * distinct[i] + nb * (8 * shapes[i][1] + 4 * shapes[i + 1][1]) for i in range(2))
    achieved = algorithmic / (count_ms * 1e-3) / 1e9
    return {"kernel": "edges_kernel<counting pass>", "bound": "hbm", "achieved": round(achieved, 1), "peak": 8000.0,
            "unit": "GB/s", "frac": round(achieved / 8000.0, 4), "traffic": None,
            "algorithmic_bytes_per_call": algorithmic, "passes_per_call": 2}


def measure_copy_gbps(torch, steps=5):
    """Device-to-device copy of 1 GiB on the current stream: the box's copy bandwidth
    (bytes read + bytes written per second)."""
    n = 1 << 28
    src = torch.arange(n, dtype=torch.int32, device="cuda:0")
    dst = torch.empty_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / steps
    del src, dst
    torch.cuda.empty_cache()
    return n * 4, ms, 2 * n * 4 / (ms * 1e-3) / 1e9


def run_oracle(oracle, og, app, B, pkw, roots_np, seed, n, first=0):
    """The oracle on roots[first : first + n]; `first` is a multiple of the sample size.
    Returns (non-NULL entries, seconds, per-step arrays)."""
    r = roots_np[first:first + n]
    base = first // pkw.get("roots_per_sample", 1)
    w = bool(pkw.get("use_weights", 0))
    t = time.perf_counter()
    if app == B.ND_KHOP:
        o = oracle.khop(og, r, pkw["fanout"], seed, sample_id_base=base, unique_rounds=pkw.get("unique_rounds", 0))
    elif app == B.ND_DEEPWALK:
        o = list(oracle.deepwalk(og, r, pkw["num_steps"], seed, use_weights=w, sample_id_base=base))
    elif app == B.ND_PPR:
        o = list(oracle.ppr(og, r, pkw["num_steps"], pkw["term_prob"], seed, use_weights=w, sample_id_base=base))
    elif app == B.ND_MULTIRW:
        o = list(oracle.multirw(og, r, pkw["roots_per_sample"], pkw["num_steps"], seed, sample_id_base=base))
    elif app == B.ND_NODE2VEC:
        o = list(oracle.node2vec(og, r, pkw["num_steps"], pkw["p"], pkw["q"], seed, use_weights=w,
                                 sample_id_base=base))
    else:
        o = oracle.layer(og, r, pkw["roots_per_sample"], pkw["fanout"], seed, sample_id_base=base, use_weights=w)
    dt = time.perf_counter() - t
    return sum(int((x >= 0).sum()) for x in o), dt, o


def run_workload(name, args, B, inputs, torch, np, cpu_baseline):
    """Times K nd_sample calls of one workload; returns the result fields of the JSON line."""
    builder, app_name, pkw, desc = WORKLOADS[name]
    app = {"deepwalk": B.ND_DEEPWALK, "ppr": B.ND_PPR, "node2vec": B.ND_NODE2VEC, "khop": B.ND_KHOP,
           "layer": B.ND_LAYER, "multirw": B.ND_MULTIRW}[app_name]
    t0 = time.time()
    g = getattr(inputs, builder)()
    if name == "c4_layer_symmetric":
        deg = np.diff(g.row_offsets).astype(np.float64)
        src = np.repeat(np.arange(g.V), np.diff(g.row_offsets))
        g.weights = (16384.0 / (deg[src] * deg[g.col_indices])).astype(np.float32)
        del src
    sys.stderr.write(f"[bench] {g.describe()} (generated in {time.time() - t0:.1f}s)\n")
    dg = B.nd_graph_create(g.row_offsets, g.col_indices, g.weights)
    if app == B.ND_LAYER:
        roots_np = inputs.permutation(g.V, 4)[:4096 * 64].copy()
    elif app == B.ND_MULTIRW:
        roots_np = inputs.permutation(g.V, 7)[:(g.V // 100) * 100].copy()
    else:
        roots_np = np.arange(g.V, dtype=np.int32)
    roots = torch.as_tensor(roots_np, device="cuda:0")
    mode = B.ND_MODE_TRANSIT_PARALLEL if args.mode == "tp" else B.ND_MODE_SAMPLE_PARALLEL
    p = B.nd_params_init(mode=mode, sched_sub_max=args.sub_max, sched_wg_max=args.wg_max,
                         lds_stage_policy=args.lds_policy,
                         sched_group_bits=args.group_bits, sched_force_class=args.force_class,
                         sched_window=args.window, **pkw)
    s = B.Sampler(dg, app, p, int(roots.numel()))
    seed = 1

    for _ in range(args.warmup):
        s.run(roots, seed)
    torch.cuda.synchronize()
    s.status()

    # Timed region: K whole nd_sample calls, bracketed by events on the launch stream.
    # Phase marks (HIP events inside the library, same stream) give the per-kernel durations
    # of the same region.
    B.nd_profile_enable(True)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    e0.record()
    marks[0].record()
    for k in range(args.steps):
        out = s.run(roots, seed)
        marks[k + 1].record()
    e1.record()
    torch.cuda.synchronize()
    ms_total = e0.elapsed_time(e1)
    per_call = sorted(marks[k].elapsed_time(marks[k + 1]) for k in range(args.steps))
    phases = B.nd_profile_read()
    B.nd_profile_enable(False)
    ms_per_step = ms_total / args.steps

    n_steps = len(s.step_len)
    slots = int(sum(s.step_len))
    live_per_step = [int((o >= 0).sum()) for o in out]
    live = int(sum(live_per_step))
    value = live / (ms_per_step * 1e-3)

    # ---- roofline of the dominant kernel: the kernel phase with the largest share of the call
    stats = s.stats() if (mode == B.ND_MODE_TRANSIT_PARALLEL and app != B.ND_LAYER) else None
    phase_ms = {k: v[0] / args.steps for k, v in phases.items() if v[1] > 0}
    launches = {k: v[1] / args.steps for k, v in phases.items() if v[1] > 0}
    kernel_phases = [k for k in ("sample_sub", "walk_window", "sample_sp", "layer", "sample_wg") if k in phase_ms]
    dom = max(kernel_phases, key=lambda k: phase_ms[k])
    avg_launch_ms = phase_ms[dom] / launches[dom]
    off_bytes = 16.0 if g.row_offsets.dtype.itemsize == 8 else 8.0        # the two row offsets of a transit
    m_per_step = [pkw["fanout"][i] if app == B.ND_KHOP else 1 for i in range(n_steps)]
    mean_deg = max(2.0, g.E / max(1, g.V))
    log_deg = float(np.ceil(np.log2(mean_deg)))
    # Algorithmic bytes of one call of the dominant kernel (what the method itself must move; an
    # adjacency entry counts 4 bytes, not the cache line it arrives in):
    #   transit-parallel, GPU-wide grouping (sample_tp_kernel): per live pair 8 (sorted transit and
    #     slot), per distinct transit the two row offsets, per non-NULL draw 4 (adjacency entry),
    #     per draw 4 (output entry).  NULL children of dead slots are written by the sort's first pass.
    #   walks grouped per window (walk_window_kernel): the pairs stay in LDS; per step and distinct
    #     transit of a window the two row offsets, per non-NULL draw 4, per sample 4 (output entry,
    #     NULL included); once per call 4 per root.  Weighted draws add 8 bytes per probe of the running
    #     sums (log2 of the mean degree probes), node2vec 4 + 4 log2(mean degree) per membership test.
    #   sample-parallel: per output entry 4, per non-NULL one 4, per parent slot 4 + (if live) two offsets.
    #   layer: per sample and transit slot 4 + two row offsets, per draw 4 + 4.
    if dom in ("sample_sub", "sample_wg") and stats is not None:
        draws = sum(int(stats[i, 0]) * m_per_step[i] for i in range(n_steps))
        total_bytes = sum(8.0 * int(stats[i, 0]) + off_bytes * int(stats[i, 1]) + 4.0 * live_per_step[i]
                          + 4.0 * int(stats[i, 0]) * m_per_step[i] for i in range(n_steps))
    elif dom == "walk_window" and stats is not None:
        draws = sum(int(stats[i, 0]) for i in range(n_steps))
        per_draw = 4.0
        if pkw.get("use_weights", 0) and app != B.ND_NODE2VEC:
            per_draw += 8.0 * log_deg
        if app == B.ND_NODE2VEC:
            per_draw += 4.0 + 4.0 * log_deg
        total_bytes = sum(off_bytes * int(stats[i, 1]) + per_draw * live_per_step[i] + 4.0 * s.step_len[i]
                          for i in range(n_steps)) + 4.0 * int(roots.numel())
        if app == B.ND_MULTIRW:                       # the picked root is read and replaced in the root sets
            total_bytes += 8.0 * draws
    elif dom == "sample_sp":
        draws = slots
        parents = [int(roots.numel())] + [int(x) for x in s.step_len[:-1]]
        live_parents = [int((roots >= 0).sum())] + live_per_step[:-1]
        total_bytes = 4.0 * slots + 4.0 * live + 4.0 * sum(parents) + off_bytes * sum(live_parents)
    else:  # layer
        draws = live
        rps = pkw["roots_per_sample"]
        n_samples = int(roots.numel()) // rps
        n_prev = [rps] + list(pkw["fanout"][:-1])
        total_bytes = n_samples * sum(n * (4.0 + off_bytes) for n in n_prev) + 8.0 * live
    alg_per_launch = total_bytes / launches[dom]
    hbm_gbs = alg_per_launch / (avg_launch_ms * 1e-3) / 1e9
    traffic = MEASURED_TRAFFIC_BYTES.get((name, args.mode, dom))
    roofline = {
        "kernel": {"sample_sub": "sample_tp_kernel", "sample_sp": "sample_sp_kernel", "layer": "layer_kernel",
                   "sample_wg": "sample_tp_kernel", "walk_window": "walk_window_kernel"}[dom],
        "bound": "hbm", "achieved": round(hbm_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": round(hbm_gbs / HBM_PEAK_GBS, 4),
        "traffic": traffic,
        "counter_frac": None if traffic is None else round(traffic / (avg_launch_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
        "overfetch": None if traffic is None else round(traffic / alg_per_launch, 3),
        "algorithmic_bytes_per_launch": int(alg_per_launch),
        "algorithmic_bytes_per_draw": round(total_bytes / max(1, draws), 2),
        "avg_launch_ms": round(avg_launch_ms, 4), "launches_per_step": launches[dom],
        "draws_per_launch": int(draws / launches[dom]),
    }

    # ---- the oracle on a prefix of the same roots: a parity check of this very run, and the CPU baseline
    import oracle
    og = oracle.OracleGraph(g.row_offsets, g.col_indices, g.weights)
    unit = pkw.get("roots_per_sample", 1)
    n_probe = min(int(roots_np.size), 2048 * unit if app != B.ND_LAYER else 2 * unit)
    live_probe, dt_probe, o_probe = run_oracle(oracle, og, app, B, pkw, roots_np, seed, n_probe)
    for i, x in enumerate(o_probe):
        got = out[i][: x.size].cpu().numpy()
        assert np.array_equal(got, np.asarray(x).reshape(-1)), f"{name}: GPU and oracle differ at step {i}"
    parity_probe = f"first {n_probe} roots, every step, equal to the oracle"
    baseline = None
    if cpu_baseline:
        n = int(min(roots_np.size, max(n_probe, n_probe * args.cpu_seconds / max(dt_probe, 1e-6))))
        n -= n % unit
        live_cpu, dt_cpu, o_single = run_oracle(oracle, og, app, B, pkw, roots_np, seed, n)
        for i, x in enumerate(o_single):     # the whole single-threaded sample against this run's GPU output
            x = np.asarray(x)
            got = out[i][: x.size].cpu().numpy()
            assert np.array_equal(got, x.reshape(-1)), f"{name}: GPU and oracle differ at step {i} (baseline sample)"
        parity_probe = f"first {n} roots, every step, equal to the oracle"
        cpu_model = ""
        try:
            with open("/proc/cpuinfo") as f:
                cpu_model = next((l.split(":", 1)[1].strip() for l in f if l.startswith("model name")), "")
        except OSError:
            pass
        baseline = {"value": round(live_cpu / dt_cpu, 1), "unit": "sampled vertices/s", "cores": 1,
                    "kind": "oracle", "cpu_model": cpu_model, "host_cpus": os.cpu_count(),
                    "sample": f"first {n} of {roots_np.size} roots of the same workload, "
                              f"{dt_cpu:.1f} s of single-threaded oracle time"}
        # The same oracle, unchanged, on disjoint ranges of the same sample from several host threads
        # (samples are independent; the C calls release the interpreter lock).  Its output must be
        # the single-threaded one.
        import concurrent.futures
        threads = max(1, min(16, os.cpu_count() or 1))
        per = (n // threads // unit) * unit
        if threads > 1 and per > 0:
            t = time.perf_counter()
            with concurrent.futures.ThreadPoolExecutor(threads) as pool:
                parts = list(pool.map(lambda k: run_oracle(oracle, og, app, B, pkw, roots_np, seed, per, k * per),
                                      range(threads)))
            dt_all = time.perf_counter() - t
            for k, (_, _, o_part) in enumerate(parts):
                for i, x in enumerate(o_part):
                    x = np.asarray(x)
                    whole = np.asarray(o_single[i])
                    if whole.ndim == 1:                       # walks: [S] per step
                        ref = whole[k * per:(k + 1) * per]
                    else:                                     # k-hop, layer: [samples, width] per step
                        ref = whole[k * per // unit:(k + 1) * per // unit]
                    assert np.array_equal(x.reshape(-1), ref.reshape(-1)), "threaded and single-threaded oracle differ"
            baseline["all_cores"] = {"value": round(sum(q[0] for q in parts) / dt_all, 1), "cores": threads,
                                     "sample": f"{threads} threads x {per} roots each (the same roots), {dt_all:.1f} s; "
                                               "output identical to the single-threaded one"}

    res = {
        "value": round(value, 1), "unit": "sampled vertices/s", "ms_per_step": round(ms_per_step, 4),
        "ms_per_call_median": round(per_call[len(per_call) // 2], 4), "ms_per_call_min": round(per_call[0], 4),
        "config": {"workload": name, "description": desc, "mode": args.mode, "group_bits": args.group_bits,
                   "window": args.window, "graph": g.describe(), "roots": int(roots.numel()), "seed": seed,
                   "slots_per_step": slots, "non_null_per_step": live},
        "slots_per_s": round(slots / (ms_per_step * 1e-3), 1),
        "phase_ms_per_step": {k: round(v, 4) for k, v in phase_ms.items()},
        "roofline": roofline, "parity_probe": parity_probe, "cpu_baseline": baseline,
    }
    if stats is not None:
        res["scheduling"] = {"live_pairs": [int(x) for x in stats[:2, 0]] + ([int(stats[-1, 0])] if len(stats) > 2 else []),
                             "distinct_transits": [int(x) for x in stats[:2, 1]],
                             "sub_wg_grid": [[int(x) for x in stats[i, 2:5]] for i in range(min(2, len(stats)))]}
    del s, out, dg
    torch.cuda.empty_cache()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default=None, choices=sorted(WORKLOADS) + ["copy_calib", "store_calib", "c4_layer_edges"],
                    help="default: c5_khop, with c5_deepwalk under \"also\"")
    ap.add_argument("--mode", default="tp", choices=["tp", "sp"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--sub-max", type=int, default=0)
    ap.add_argument("--wg-max", type=int, default=0)
    ap.add_argument("--group-bits", type=int, default=0,
                    help="0: exact transit grouping (default); b: group by the top b bits of the vertex id only")
    ap.add_argument("--window", type=int, default=0,
                    help="walks: 0 windows of samples in LDS (default), -1 GPU-wide grouping, 1024 / 2048 window size")
    ap.add_argument("--lds-policy", type=int, default=0, choices=[0, 1, 2],
                    help="ablation: 0 stage adjacency lists in LDS where it pays (default), 1 never, 2 whenever they fit")
    ap.add_argument("--force-class", type=int, default=-1,
                    help="ablation: -1 balanced (default), 0/1/2 every transit sub-wavefront/workgroup/grid")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only; sampling shards by samples with the "
              "graph replicated, which one GPU cannot show (use --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2009_06693_amd import binding as B
    from paper_2009_06693_amd import inputs

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.workload == "copy_calib":
        # A plain device-to-device copy of known size: the yardstick that turns the
        # FETCH_SIZE / WRITE_SIZE counters of a profiler run into bytes.
        nbytes, ms, gbps = measure_copy_gbps(torch, args.steps)
        print(json.dumps({"workload": "copy_calib", "bytes_read": nbytes, "bytes_written": nbytes,
                          "ms_per_copy": round(ms, 4), "copy_GBps": round(gbps, 1)}))
        return
    if args.workload == "store_calib":
        # What scattered stores cost on this GPU: runs of run_len ints at scattered run-aligned places
        # of a 2.7 GB array against whole 128-byte lines at scattered places and against stores in order.
        n_runs = 1 << 26
        buf = torch.empty(n_runs * 10, dtype=torch.int32, device="cuda:0")
        rows = []
        for what, runs, run_len, scattered in (("40-byte runs (10 ints), scattered", n_runs, 10, True),
                                               ("4-byte runs, scattered", n_runs, 1, True),
                                               ("64-byte runs (16 ints), scattered", 1 << 25, 16, True),
                                               ("whole 128-byte lines (32 ints), scattered", 1 << 24, 32, True),
                                               ("40-byte runs in order", n_runs, 10, False),
                                               ("40-byte runs, scattered inside 16 windows of 168 MB, one launch per window",
                                                n_runs, 10, 16),
                                               ("40-byte runs, scattered inside 64 windows of 42 MB, one launch per window",
                                                n_runs, 10, 64)):
            def go():
                if scattered is True or scattered is False:
                    B.nd_probe_store_runs(buf, runs, run_len, scattered)
                else:                                    # `scattered` windows, each its own launch
                    per = runs // scattered
                    for w in range(scattered):
                        B.nd_probe_store_runs(buf[w * per * run_len:(w + 1) * per * run_len], per, run_len, True)
            go()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(args.steps):
                go()
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / args.steps
            rows.append({"pattern": what, "runs": runs, "ms": round(ms, 4), "runs_per_s": round(runs / (ms * 1e-3), 1),
                         "payload_GBps": round(runs * run_len * 4 / (ms * 1e-3) / 1e9, 1)})
        print(json.dumps({"workload": "store_calib", "patterns": rows}))
        return
    if args.workload == "c4_layer_edges":
        return bench_layer_edges(args, B, inputs, torch, np)

    primary = args.workload or "c5_khop"
    res = run_workload(primary, args, B, inputs, torch, np, cpu_baseline=not args.no_cpu_baseline)
    also = None
    if args.workload is None:
        also = run_workload("c5_deepwalk", args, B, inputs, torch, np, cpu_baseline=False)
    _, _, copy_gbps = measure_copy_gbps(torch)
    res["roofline"]["copy_GBps"] = round(copy_gbps, 1)
    line = {
        "metric": "sampled vertices/sec per step-batch on 1 MI355X; achieved HBM GB/s vs peak",
        "value": res["value"], "unit": res["unit"], "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": res["ms_per_step"], "ms_per_call_median": res["ms_per_call_median"],
        "ms_per_call_min": res["ms_per_call_min"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "int32", "data": "synthetic",
    }
    for k in ("config", "slots_per_s", "phase_ms_per_step", "roofline", "parity_probe", "cpu_baseline", "scheduling"):
        if k in res:
            line[k] = res[k]
    if also is not None:
        also["roofline"]["copy_GBps"] = round(copy_gbps, 1)
        also.pop("cpu_baseline", None)
        line["also"] = also
    print(json.dumps(line))


if __name__ == "__main__":
    main()
