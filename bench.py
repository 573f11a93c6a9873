"""Benchmark of the planning hot path on one MI355X.

A step is one pass of the whole path over one synthetic trace and its candidate
orders, all inputs already resident in device memory (the orders are produced on
the device by stalloc_make_orders before the timed region):
    stalloc_plan (all P orders, best plan kept)
 -> stalloc_validate (the best plan, all pairs)
 -> stalloc_lower_bound.
The default workload is the largest configuration (interleaved 1F1B trace, 199 748
requests, 4096 orders).  The headline value is placed requests x plans per second,
n * P * steps / time.

Prints ONE JSON line.  `roofline` describes the dominant kernel (the placement
kernel).  Algorithmic work per launch: 28 B of HBM per placement (order entry,
request record, address written); one stored block record and 8 integer lane
operations per lifetime-overlapping pair and plan.  The floor that takes longest
at the chip's peak names the bound; achieved = that work / time of the
stalloc_plan call measured with events on the launch stream (the placement kernel
is all but a fraction of a millisecond of it).  `peak_measured` / `frac_measured`
set the same work against what plain probe kernels reach on this very device.
`traffic` holds HBM-side bytes per launch from rocprofv3 counter runs, and is null
unless those runs were made with the kernel sources as they are now.
`cpu_baseline` is the CPU oracle timed on a bounded sample of the same workload on
this machine's host cores: one thread on a fixed few orders, and all threads.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PER_PLACEMENT_BYTES = 28    # 4 B order entry + 16 B request record + 8 B address written
OPS_PER_CANDIDATE = 8       # 2 lifetime compares, and, select, running max, add, compare, and
LDS_PEAK_GBS = 256 * 128 * 2.4          # 256 CUs x 128 B/clk x 2.4 GHz = 78 643 GB/s
HBM_PEAK_GBS = 8000.0
ALU_PEAK_TOPS = 256 * 64 * 2.4e9 / 1e12  # 256 CUs x 64 integer lanes x 2.4 GHz = 39.3 T lane-ops/s
KERNEL_NAMES = {"bitmap": "plan_bitmap_kernel", "list_lds": "plan_kernel", "list_memory": "plan_kernel",
                "long_list": "plan_split_kernel"}

# HBM-side bytes per launch of the placement kernel, from two rocprofv3 --pmc runs of this script
# (FETCH_SIZE and WRITE_SIZE in KiB, each scaled by what the same counter reads for a plain copy of
# known size in the same run; the summaries are under profiles/).  Keyed by (configuration, orders);
# each entry names the sources of stalloc_plan it was measured with (source_digest() below): with any
# other sources the figure is not reported.
MEASURED_TRAFFIC = {(5, 4096): {"bytes": (269_114_935 * 2 + 102_024_208) * 1024, "sources": "dcab51237f78c6bb"}}


# The sources stalloc_plan and its kernels are built from (the other entry points have files of their own).
PLAN_SOURCES = ("plan.hip", "plan_split.hip", "plan_bitmap.hip", "plan_list.h", "plan_params.h", "host_util.h", "wave.h",
                "sort_keys.h", "trace_check.hip", "orders.hip", "layers.hip")


def source_digest() -> str:
    """SHA-256 over the sources of stalloc_plan and its kernels (csrc/, by name)."""
    h = hashlib.sha256()
    for name in sorted(PLAN_SOURCES):
        h.update(name.encode())
        h.update(open(os.path.join(ROOT, "paper_2507_16274_amd", "csrc", name), "rb").read())
    return h.hexdigest()[:16]


def measured_peaks(S, torch) -> dict:
    """What plain probe kernels reach on this device: copy (GB/s read + written), LDS reads, integer lanes."""
    out = {}
    buf = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
    for name, what, iters, scale in (("hbm_copy_GBs", 0, 0, 1e9), ("lds_read_GBs", 1, 4096, 1e9), ("int_alu_TOPS", 2, 4096, 1e12)):
        best = 0.0
        for _ in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            work = S.stalloc_probe(what, buf, iters)
            e1.record()
            torch.cuda.synchronize()
            best = max(best, work / (e0.elapsed_time(e1) * 1e-3) / scale)
        out[name] = best
    del buf
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=5, help="trace configuration 1..5, or 6..7 for the second kind of workload (default: 5)")
    ap.add_argument("--plans", type=int, default=0, help="override the number of orders (0 = the configuration's)")
    ap.add_argument("--cpu-seconds", type=float, default=25.0, help="CPU work budget of each leg of the oracle baseline")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-offsets", action="store_true", help="do not have the addresses of all plans written (only extents and the best plan)")
    ap.add_argument("--reusable", type=int, default=0, metavar="K",
                    help="also time stalloc_reusable_space for K windows over the best plan (reported beside the step)")
    ap.add_argument("--checks", action="store_true",
                    help="also time stalloc_validate (all plans; the best plan alone) and stalloc_lower_bound in timed "
                         "regions of their own (reported beside the step)")
    ap.add_argument("--graph", action="store_true",
                    help="also capture one step in a graph and time its replays (the calls allocate nothing and use "
                         "the caller's stream only)")
    ap.add_argument("--make-orders", action="store_true",
                    help="also time the production of the run's orders on the device (stalloc_make_orders) and compare "
                         "sampled rows with the host's arrays")
    ap.add_argument("--layers", action="store_true",
                    help="also build the memory-layers of the trace (Algorithm 1), plan the layers under as many "
                         "orders and expand the plans to the requests, in a timed region of its own")
    ap.add_argument("--fusion", action="store_true",
                    help="also fuse every candidate pair of HomoPhase groups of the trace (Sec. 5.1) in a timed region "
                         "of its own")
    ap.add_argument("--copy-calibration-mib", type=int, default=0,
                    help="also run one plain device copy of this many MiB (reference dispatch for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: exactly one GPU is supported (orders are independent and would be split "
              "across GPUs, but no multi-GPU path exists); use --gpus 1", file=sys.stderr)
        return 2

    import torch
    import paper_2507_16274_amd as S
    from workloads import CONFIGS, make_orderings, make_trace, trace_stats

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)

    cfg = CONFIGS[args.config]
    tr = make_trace(args.config)
    stats = trace_stats(tr)
    P = args.plans or cfg.n_orderings
    n = tr.n

    size, ta, tf = S.trace_to_device(tr)
    made = S.stalloc_make_orders(size, ta, tf, tr.t_end, P)          # rows 0 .. P-1 of the family, seed 1000
    torch.cuda.synchronize()
    S.check_status(made, "stalloc_make_orders")
    orders = made["orders"]
    del made
    # the rows the CPU legs and the consistency checks look at, made on the host as well
    sample_rows = np.unique(np.r_[0, 1, 2, np.linspace(0, P - 1, 61).astype(np.int64)])
    host_rows = make_orderings(tr, P, rows=sample_rows)
    if not np.array_equal(orders[torch.from_numpy(sample_rows).cuda()].cpu().numpy().view(np.uint32), host_rows):
        print("bench.py: orders made on the device differ from the host's", file=sys.stderr)
        return 1
    cache_plan, cache_val, cache_lb = {}, {}, {}
    outs = {"offsets": None if args.no_offsets else torch.empty((P, n), dtype=torch.int64, device="cuda"),
            "peaks": torch.empty(P, dtype=torch.int64, device="cuda"),
            "best_offsets": torch.empty(n, dtype=torch.int64, device="cuda"),
            "best_plan": torch.empty(1, dtype=torch.int32, device="cuda"),
            "status": torch.empty(1, dtype=torch.int32, device="cuda")}

    ev_pairs = []

    def step(timed: bool):
        if timed:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
        plan = S.stalloc_plan(size, ta, tf, tr.t_end, orders, out=outs, workspace_cache=cache_plan,
                              want_offsets=not args.no_offsets)
        if timed:
            e1.record()
            ev_pairs.append((e0, e1))
        val = S.stalloc_validate(size, ta, tf, tr.t_end, plan["best_offsets"].view(1, n), workspace_cache=cache_val)
        lb = S.stalloc_lower_bound(size, ta, tf, tr.t_end, workspace_cache=cache_lb)
        return plan, val, lb

    if args.copy_calibration_mib:
        src = torch.ones(args.copy_calibration_mib * 2 ** 20 // 4, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        plan, val, lb = step(True)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    S.check_status(plan, "stalloc_plan")
    S.check_status(val, "stalloc_validate")
    S.check_status(lb, "stalloc_lower_bound")
    conflicts = int(val["conflicts"].item())
    lower_bound = int(lb["lower_bound"].item())
    peaks = plan["peaks"].cpu().numpy().view(np.uint64)
    best = int(plan["best_plan"].item())
    best_peak = int(peaks[best])
    if conflicts != 0 or best_peak < lower_bound or best_peak != int(peaks.min()):
        print(f"bench.py: inconsistent result (conflicts={conflicts}, best={best_peak}, lb={lower_bound})", file=sys.stderr)
        return 1

    ms_per_step = elapsed / args.steps * 1e3
    value = n * P * args.steps / elapsed
    plan_ms = float(np.mean([a.elapsed_time(b) for a, b in ev_pairs]))
    # which kernel placed the trace and how it stores a placed block (decided on the device)
    info = S.stalloc_plan_report(plan)
    in_lds = info["kernel"] != "list_memory"
    entry_bytes = {"bitmap": 4, "long_list": info["list_entry_bytes"] or 16}.get(info["kernel"], {16: 8, 32: 16, 64: 24}.get(info["address_bits"], 24))
    pairs = stats["E"] * P                       # lifetime-overlapping (earlier, later) pairs examined at least once
    t_s = plan_ms * 1e-3
    hbm_bytes = PER_PLACEMENT_BYTES * n * P
    state_bytes = entry_bytes * pairs
    algo_ops = OPS_PER_CANDIDATE * pairs
    # the three floors: mandatory HBM stream, stored-block traffic, integer ALU work; the largest one binds
    floors = {"hbm": hbm_bytes / (HBM_PEAK_GBS * 1e9),
              "lds" if in_lds else "hbm_list": state_bytes / ((LDS_PEAK_GBS if in_lds else HBM_PEAK_GBS) * 1e9),
              "alu": algo_ops / (ALU_PEAK_TOPS * 1e12)}
    bound = max(floors, key=floors.get)
    if in_lds and floors["alu"] >= floors["lds"] * 0.999:
        bound = "alu"                            # (16-byte records at the LDS rate and 8 lane operations take the same time)
    kernel = KERNEL_NAMES.get(info["kernel"], info["kernel"])
    peaks_here = measured_peaks(S, torch)
    result = {
        "metric": "placed requests x plans / s",
        "value": value,
        "unit": "requests*plans/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u64" if info["address_bits"] == 64 else "u32",
        "data": "synthetic",
        "config": {"workload": (f"configs[{args.config - 1}] " if args.config <= 5 else "second workload ") +
                               f"{cfg.name}: {cfg.description}", "n": n, "P": P,
                   "T": stats["T"], "E": stats["E"], "distinct_sizes": stats["distinct_sizes"],
                   "orders": "stalloc_make_orders on the device, before the timed region",
                   "step": "stalloc_plan(all orders) + stalloc_validate(best plan) + stalloc_lower_bound"},
        "quality": {"lower_bound": lower_bound, "best_peak": best_peak, "best_plan": best,
                    "lower_bound_over_peak": lower_bound / best_peak,
                    "median_lower_bound_over_peak": float(lower_bound / np.median(peaks.astype(np.float64)))},
    }
    if bound == "alu":
        roof = {"bound": "alu", "kernel": kernel, "achieved": algo_ops / t_s / 1e12, "peak": ALU_PEAK_TOPS, "unit": "TOP/s",
                "frac": algo_ops / t_s / 1e12 / ALU_PEAK_TOPS, "peak_measured": peaks_here["int_alu_TOPS"],
                "frac_measured": algo_ops / t_s / 1e12 / peaks_here["int_alu_TOPS"]}
    elif not in_lds:
        roof = {"bound": "hbm", "kernel": kernel, "achieved": (hbm_bytes + state_bytes) / t_s / 1e9, "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": (hbm_bytes + state_bytes) / t_s / 1e9 / HBM_PEAK_GBS,
                "peak_measured": peaks_here["hbm_copy_GBs"],
                "frac_measured": (hbm_bytes + state_bytes) / t_s / 1e9 / peaks_here["hbm_copy_GBs"]}
    else:
        roof = {"bound": "lds", "kernel": kernel, "achieved": state_bytes / t_s / 1e9, "peak": LDS_PEAK_GBS, "unit": "GB/s",
                "frac": state_bytes / t_s / 1e9 / LDS_PEAK_GBS, "peak_measured": peaks_here["lds_read_GBs"],
                "frac_measured": state_bytes / t_s / 1e9 / peaks_here["lds_read_GBs"]}
    digest = source_digest()
    traffic = MEASURED_TRAFFIC.get((args.config, P))
    roof.update({
        "traffic": traffic["bytes"] if traffic and traffic["sources"] == digest else None,
        "kernel_ms": plan_ms, "placement_kernel": info["kernel"], "stored_block_bytes": entry_bytes, "blocks_in_lds": in_lds,
        "lifetime_threshold": info["lifetime_threshold"], "long_requests": info["long_requests"],
        "large_short_lived_from_bytes": info["large_size"], "large_short_lived_requests": info["large_requests"],
        "plans_placed_again_with_64_bit_addresses": info["plans_64bit"],
        "algorithmic_ops": algo_ops, "algorithmic_list_bytes": state_bytes, "algorithmic_hbm_bytes": hbm_bytes,
        "floor_ms": {k: v * 1e3 for k, v in floors.items()},
        "hbm_stream_GBs": hbm_bytes / t_s / 1e9, "list_GBs": state_bytes / t_s / 1e9,
        "measured_on_this_device": peaks_here, "kernel_sources": digest})
    result["roofline"] = roof

    if args.reusable:
        # Dynamic reusable space of the best plan (Sec. 5.2) for K layer-like windows: its own timed
        # region.  Algorithmic work: every window looks at every decision once: 8 lane operations (two
        # compares, select, 64-bit running maximum, compare).  The 24 B of a decision (address range,
        # lifespan) serve many windows at once, so the bytes that must move are the plan, the windows
        # and the answers only; the figure for one read per window is kept for comparison.
        from workloads import make_windows
        K = args.reusable
        windows_np = make_windows(tr, K, seed=7000 + args.config)
        windows = torch.from_numpy(windows_np.view(np.int32)).cuda()
        cap, cache_rs = 64, {}
        best_offsets = plan["best_offsets"].clone()
        for _ in range(args.warmup):
            S.stalloc_reusable_space(size, ta, tf, tr.t_end, best_offsets, windows, cap, workspace_cache=cache_rs)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            rs = S.stalloc_reusable_space(size, ta, tf, tr.t_end, best_offsets, windows, cap, workspace_cache=cache_rs)
        e1.record()
        torch.cuda.synchronize()
        S.check_status(rs, "stalloc_reusable_space")
        rs_ms = e0.elapsed_time(e1) / args.steps
        rs_bytes, rs_ops = 24 * n * K, 8 * n * K
        mean_intervals = float(rs["counts"].float().mean().item())
        must_move = 24 * n + 8 * K + K * (12 + 16 * min(mean_intervals, cap))
        result["reusable_space"] = {
            "windows": K, "ms_per_call": rs_ms, "windows_per_s": K / (rs_ms * 1e-3),
            "mean_intervals": mean_intervals,
            "roofline": {"bound": "alu", "kernel": "rs_sweep / rs_sweep_by_window (+ sort, rs_gather)",
                         "achieved": rs_ops / (rs_ms * 1e-3) / 1e12, "peak": ALU_PEAK_TOPS, "unit": "TOP/s",
                         "frac": rs_ops / (rs_ms * 1e-3) / 1e12 / ALU_PEAK_TOPS,
                         "traffic": None, "algorithmic_ops": rs_ops, "algorithmic_bytes": must_move,
                         "one_read_per_window_GBs": rs_bytes / (rs_ms * 1e-3) / 1e9,
                         "floor_ms": {"hbm": must_move / (HBM_PEAK_GBS * 1e9) * 1e3, "alu": rs_ops / (ALU_PEAK_TOPS * 1e12) * 1e3}}}
        if not args.no_cpu_baseline:
            import oracle
            oracle.build()
            sample = min(K, 64)
            t1 = time.perf_counter()
            best_np = best_offsets.cpu().numpy().view(np.uint64)
            counts = rs["counts"].cpu().numpy()
            for w in range(sample):
                _, c, _ = oracle.reusable_space(tr.size, tr.t_alloc, tr.t_free, best_np,
                                                (int(windows_np[w, 0]), int(windows_np[w, 1])), cap=cap)
                if c != int(counts[w]):
                    print("bench.py: reusable-space counts differ from the oracle", file=sys.stderr)
                    return 1
            wall = time.perf_counter() - t1
            result["reusable_space"]["cpu_baseline"] = {"value": sample / wall, "unit": "windows/s", "cores": 1,
                                                        "kind": "oracle", "sample": f"first {sample} windows"}

    if args.graph:
        # One step captured once and replayed: the ~30 launches of a step cost no host time any more.
        g_stream = torch.cuda.Stream()
        g_stream.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(g_stream):
            step(False)
            g_stream.synchronize()
            with torch.cuda.graph(graph, stream=g_stream):
                g_plan, g_val, g_lb = step(False)
        torch.cuda.current_stream().wait_stream(g_stream)
        for _ in range(max(args.warmup, 1)):
            graph.replay()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        g_elapsed = time.perf_counter() - t1
        if not torch.equal(g_plan["peaks"], plan["peaks"]) or int(g_val["conflicts"].item()) != 0 or \
                int(g_lb["lower_bound"].item()) != lower_bound:
            print("bench.py: the replayed step differs from the eager one", file=sys.stderr)
            return 1
        result["graph"] = {"ms_per_step": g_elapsed / args.steps * 1e3, "value": n * P * args.steps / g_elapsed}

    if args.make_orders:
        # The orders of this run produced on the device: P rows of n keys sorted.  What must move is the
        # result (4 B per entry); the sort itself writes 16-byte keys once per pass (log2(n / 256) + 1 passes).
        cache_o = {}
        for _ in range(max(args.warmup, 1)):
            made = S.stalloc_make_orders(size, ta, tf, tr.t_end, P, workspace_cache=cache_o)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            made = S.stalloc_make_orders(size, ta, tf, tr.t_end, P, workspace_cache=cache_o)
        e1.record()
        torch.cuda.synchronize()
        S.check_status(made, "stalloc_make_orders")
        if not torch.equal(made["orders"], orders):
            print("bench.py: two runs of stalloc_make_orders differ", file=sys.stderr)
            return 1
        mo_ms = e0.elapsed_time(e1) / args.steps
        passes = 1 + max(0, int(np.ceil(np.log2(max(1, -(-n // 256))))))
        result["make_orders"] = {
            "ms_per_call": mo_ms, "keys_per_s": n * P / (mo_ms * 1e-3), "sort_passes": passes,
            "roofline": {"bound": "hbm", "kernel": "or_sort_tiles + or_merge passes + or_emit",
                         "achieved": 4 * n * P / (mo_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": 4 * n * P / (mo_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "traffic": None,
                         "algorithmic_bytes": 4 * n * P,
                         "sort_buffer_GBs": (32 * passes + 4) * n * P / (mo_ms * 1e-3) / 1e9}}

    if args.fusion:
        # HomoPhase groups (requests allocated in one phase and released in one other phase) and every pair of
        # them in which one is released in the phase the other is allocated in: one workgroup per pair, a
        # chain of placement steps inside (bound by that chain, not by bytes or lane operations).
        from workloads.groups import candidate_pairs, flatten_pairs
        groups, pairs = candidate_pairs(tr.p_alloc, tr.p_free)
        members, begin, count1, largest = flatten_pairs(groups, pairs)
        dev = lambda a: torch.from_numpy(np.ascontiguousarray(a).view(np.int32)).cuda()
        d_members, d_begin, d_count1 = dev(members), dev(begin), dev(count1)
        cache_f = {}
        fuse = lambda: S.stalloc_fuse_groups(size, ta, tf, tr.t_end, d_members, d_begin, d_count1, largest, workspace_cache=cache_f)
        for _ in range(max(args.warmup, 1)):
            fuse()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            f = fuse()
        e1.record()
        torch.cuda.synchronize()
        S.check_status(f, "stalloc_fuse_groups")
        f_acc, f_ext = f["accepted"].cpu().numpy(), f["extents"].cpu().numpy().view(np.uint64)
        if (f_ext[:, 2] > f_ext[:, 0] + f_ext[:, 1]).any() or (f_ext[:, 2] < np.maximum(f_ext[:, 0], f_ext[:, 1])).any():
            print("bench.py: a fused plan is larger than its two plans stacked, or smaller than the larger of them", file=sys.stderr)
            return 1
        result["fusion"] = {"groups": len(groups), "pairs": len(pairs), "requests_in_pairs": int(len(members)),
                            "largest_pair": largest, "accepted": int(f_acc.sum()), "ms_per_call": e0.elapsed_time(e1) / args.steps}

    if args.layers:
        # HomoSize groups -> memory-layers (Sec. 5.1, Algorithm 1), each layer planned as one request under
        # P orders of the layers, the plans expanded to the requests and the best one validated.  The
        # construction is sequential inside a group (one wave per group), so it is bound by the chain of
        # dependent steps of the longest group, not by bytes or lane operations.
        from workloads import Trace
        cache_ly, cache_lp, cache_lv = {}, {}, {}
        ly = S.stalloc_memory_layers(size, ta, tf, tr.t_end, workspace_cache=cache_ly)
        torch.cuda.synchronize()
        S.check_status(ly, "stalloc_memory_layers")
        L = int(ly["n_layers"].item())
        l_size, l_ta, l_tf = ly["layer_size"][:L].clone(), ly["layer_t_alloc"][:L].clone(), ly["layer_t_free"][:L].clone()
        ltr = Trace(name="layers", size=l_size.cpu().numpy().view(np.uint64), t_alloc=l_ta.cpu().numpy().view(np.uint32),
                    t_free=l_tf.cpu().numpy().view(np.uint32), t_end=tr.t_end)
        l_orders = torch.from_numpy(make_orderings(ltr, min(P, 1024)).view(np.int32)).cuda()

        def layer_family():
            a = S.stalloc_memory_layers(size, ta, tf, tr.t_end, workspace_cache=cache_ly)
            b = S.stalloc_plan(l_size, l_ta, l_tf, tr.t_end, l_orders, workspace_cache=cache_lp)
            c = S.stalloc_expand_layers(a["layer_of"], b["offsets"])
            return a, b, c

        for _ in range(max(args.warmup, 1)):
            layer_family()
        torch.cuda.synchronize()
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
        evs[0].record()
        for _ in range(args.steps):
            a = S.stalloc_memory_layers(size, ta, tf, tr.t_end, workspace_cache=cache_ly)
        evs[1].record()
        for _ in range(args.steps):
            b = S.stalloc_plan(l_size, l_ta, l_tf, tr.t_end, l_orders, workspace_cache=cache_lp)
        evs[2].record()
        for _ in range(args.steps):
            c = S.stalloc_expand_layers(a["layer_of"], b["offsets"])
        evs[3].record()
        torch.cuda.synchronize()
        S.check_status(b, "stalloc_plan(layers)")
        S.check_status(c, "stalloc_expand_layers")
        l_peaks = b["peaks"].cpu().numpy().view(np.uint64)
        l_best = int(b["best_plan"].item())
        v = S.stalloc_validate(size, ta, tf, tr.t_end, c["offsets"][l_best].view(1, n).contiguous(), workspace_cache=cache_lv)
        torch.cuda.synchronize()
        if int(v["conflicts"].item()) != 0 or int(l_peaks[l_best]) < lower_bound:
            print("bench.py: the expanded layer plan is not a valid plan", file=sys.stderr)
            return 1
        ms = [evs[i].elapsed_time(evs[i + 1]) / args.steps for i in range(3)]
        result["layers"] = {
            "n_layers": L, "orders": P,
            "ms_memory_layers": ms[0], "requests_per_s": n / (ms[0] * 1e-3),
            "ms_plan_layers": ms[1], "layer_plans_per_s": L * P / (ms[1] * 1e-3),
            "ms_expand": ms[2], "expand_GBs": (12 * n * P) / (ms[2] * 1e-3) / 1e9,
            "best_peak": int(l_peaks[l_best]), "lower_bound_over_peak": lower_bound / int(l_peaks[l_best]),
            "per_request_best_lower_bound_over_peak": lower_bound / best_peak}

    if args.checks:
        # The two checking calls in timed regions of their own.  stalloc_validate tests every unordered
        # pair of a plan: 4 compares, 3 ands and a count = 8 lane operations per pair; its bytes (24 per
        # request and tile pass) are negligible.  stalloc_lower_bound streams the trace (16 B per request),
        # scatters two 8-byte sums per request and passes twice over 8 B per timestamp.
        def timed(fn):
            for _ in range(max(args.warmup, 1)):
                fn()
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(args.steps):
                out = fn()
            b.record()
            torch.cuda.synchronize()
            return out, a.elapsed_time(b) / args.steps

        def pair_roofline(plans, ms):
            ops = 8 * (n * (n - 1) // 2) * plans
            return {"plans": plans, "ms_per_call": ms, "pairs_per_s": ops / 8 / (ms * 1e-3),
                    "roofline": {"bound": "alu", "kernel": "val_pairs", "achieved": ops / (ms * 1e-3) / 1e12,
                                 "peak": ALU_PEAK_TOPS, "unit": "TOP/s", "frac": ops / (ms * 1e-3) / 1e12 / ALU_PEAK_TOPS,
                                 "traffic": None, "algorithmic_ops": ops}}

        cache_all, cache_one, cache_l = {}, {}, {}
        best_row = plan["best_offsets"].clone().view(1, n)
        all_rows = plan["offsets"].clone()
        v_all, ms_all = timed(lambda: S.stalloc_validate(size, ta, tf, tr.t_end, all_rows, workspace_cache=cache_all))
        v_one, ms_one = timed(lambda: S.stalloc_validate(size, ta, tf, tr.t_end, best_row, workspace_cache=cache_one))
        l_out, ms_lb = timed(lambda: S.stalloc_lower_bound(size, ta, tf, tr.t_end, workspace_cache=cache_l))
        cache_t = {}
        t_out, ms_tmp = timed(lambda: S.stalloc_tmp(size, ta, tf, tr.t_end, plan["peaks"], workspace_cache=cache_t))
        S.check_status(t_out, "stalloc_tmp")
        tmp_all = t_out["tmp"].cpu().numpy()
        S.check_status(v_all, "stalloc_validate")
        S.check_status(v_one, "stalloc_validate")
        S.check_status(l_out, "stalloc_lower_bound")
        if int(v_all["conflicts"].sum().item()) != 0 or int(v_one["conflicts"].item()) != 0:
            print("bench.py: a plan has conflicts", file=sys.stderr)
            return 1
        lb_bytes = 32 * n + 16 * stats["T"]
        result["quality"]["tmp_best_plan"] = float(tmp_all[best])          # Eq. 2 over the whole plan
        result["quality"]["tmp_median"] = float(np.median(tmp_all))
        result["checks"] = {
            "tmp_all_plans": {"ms_per_call": ms_tmp, "algorithmic_bytes": 16 * n + 16 * P},
            "validate_all_plans": pair_roofline(P, ms_all),
            "validate_best_plan": pair_roofline(1, ms_one),
            "lower_bound": {"ms_per_call": ms_lb,
                            "roofline": {"bound": "hbm", "kernel": "lb_clear, lb_scatter, lb_tiles", "achieved": lb_bytes / (ms_lb * 1e-3) / 1e9,
                                         "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": lb_bytes / (ms_lb * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                         "traffic": None, "algorithmic_bytes": lb_bytes}}}

    if not args.no_cpu_baseline:
        # The oracle as it stands (conflict-list method) on this machine's host cores, on rows the host made
        # itself: (a) one thread on a fixed few rows, (b) all threads on evenly spaced rows; each leg is cut to
        # about --cpu-seconds of work, judged by the time the first row takes.  Every extent is compared.
        import oracle
        oracle.build()
        cores = min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", "0")) or (os.cpu_count() or 1))
        t1 = time.perf_counter()
        lists = oracle.conflict_lists(tr.t_alloc, tr.t_free)
        lists_s = time.perf_counter() - t1
        t1 = time.perf_counter()
        _, e_first = oracle.plan_lists(tr.size, lists, host_rows[0])
        one = time.perf_counter() - t1
        single_rows = int(max(1, min(8, len(sample_rows), args.cpu_seconds / max(one, 1e-6))))
        t1 = time.perf_counter()
        a_cpu, e_single = oracle.plan_many(tr.size, tr.t_alloc, tr.t_free, host_rows[:single_rows], threads=1,
                                           method="lists", lists=lists)
        single_wall = time.perf_counter() - t1
        # (whole rounds of one row per thread; side by side the rows take about twice as long as the first one alone)
        many = int(max(1, min(len(sample_rows), cores * max(1, int(args.cpu_seconds / max(2.2 * one, 1e-6))))))
        pick = np.linspace(0, len(sample_rows) - 1, many).astype(np.int64)
        t1 = time.perf_counter()
        a_cpu, e_cpu = oracle.plan_many(tr.size, tr.t_alloc, tr.t_free, host_rows[pick], threads=cores,
                                        method="lists", lists=lists)
        wall = time.perf_counter() - t1
        if not np.array_equal(e_cpu, peaks[sample_rows[pick]]) or not np.array_equal(e_single, peaks[sample_rows[:single_rows]]):
            print("bench.py: GPU extents differ from the oracle on the baseline sample", file=sys.stderr)
            return 1
        result["cpu_baseline"] = {"value": n * many / wall, "unit": "requests*plans/s", "cores": cores, "kind": "oracle",
                                  "sample": f"{many} of {P} orders (evenly spaced among rows 0-2 and 61 spread rows), conflict-list "
                                            f"oracle, {wall:.2f} s wall on {cores} threads; its lists of lifetime-conflicting "
                                            f"requests took {lists_s:.2f} s once (not counted)",
                                  "single_thread": {"value": n * single_rows / single_wall, "unit": "requests*plans/s", "cores": 1,
                                                    "sample": f"the first {single_rows} of those rows, {single_wall:.2f} s"}}
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
