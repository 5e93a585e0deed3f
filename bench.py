#!/usr/bin/env python3
"""Benchmark of the K-hop precompute on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload all|1..5]

One step = one gp_propagate call: the whole hot path (slot-0 copy, K hops of
gather/scale/accumulate over all edge blocks, completion of cut rows) on one
synthetic workload whose inputs already sit in HBM.  Prints ONE JSON line:
throughput in giga edge-feature updates per second (nnz * d * K / t / 1e9), the
HBM roofline of the dominant kernel (algorithmic bytes per launch over the
kernel's mean duration, timed with HIP events on the launch stream), and the CPU
oracle timed beside it on the host cores as a baseline.

The default times all four in-HBM workloads; the line is the one of the largest
(config 4) and carries the others under "other_workloads".
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0

FP32_VECTOR_PEAK_TFLOPS = 157.3
LDS_PEAK_GBS = 256 * 256 * 2.4   # 256 compute units x 256 bytes per clock (ds_read_b128, measured: 146 TB/s sequential) x 2.4 GHz
HEADLINE_WORKLOAD = 4            # the largest workload that is resident in HBM
IN_HBM_WORKLOADS = (1, 2, 3, 4)

# HBM bytes per launch of the dominant kernel as the last counter run recorded them
# (bench_counters.py: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE passes over this script, each
# scaled by what the same counter reads for the library's plain copy kernel).  The figure is
# reported only when it was recorded for the same workload and library options.
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hop_traffic.json")


def recorded_traffic(workload: int, options: dict):
    try:
        with open(TRAFFIC_FILE) as f:
            rec = json.load(f).get(str(workload))
    except (OSError, ValueError):
        return None
    if not rec or rec.get("options") != options:
        return None
    return rec

WORKLOAD_NAMES = {
    1: "config1: G(n,M) 10k nodes / 210k nnz, d=128 fp32, sym, K=2, 4 edge blocks",
    2: "config2: Chung-Lu 169,343 nodes / ~2.5M nnz, d=128 fp32, sym, K=3",
    3: "config3: Chung-Lu 2.45M nodes / ~123M nnz, d=100 fp32, mean, K=3, 8M-edge blocks",
    4: "config4: SBM 233k nodes / ~114M nnz, d=602 fp32, sum, K=2",
    5: "config5: Chung-Lu 111M nodes / ~3.3B nnz, d=128 bf16 storage, sym, K=3, out-of-core",
}


def algorithmic_bytes_per_hop(n: int, nnz: int, d: int, elem: int) -> int:
    """Compulsory traffic of one hop: column ids (4 B per non-zero), the int64 row
    pointers, one fp32 normalisation vector, X_{k-1} read once, X_k written once."""
    return 4 * nnz + 8 * (n + 1) + 4 * n + 2 * n * d * elem


LC_WIDTHS = [256, 256, 256, 40]      # hidden 256 (Appendix B), four MLP layers (GPRGNN's setting), 40 classes
MFMA_F32_PEAK_TFLOPS = 157.3


def bench_lc(args, gp, torch, w, plan, stack, t_gen, t_plan, cpu_baseline=True):
    """One step = the LC-version forward pass (Appendix A) over all n rows of the hop
    stack gp_propagate left in HBM, in mini-batches of --lc-batch randomly permuted
    rows (the paper trains with batches of 4096)."""
    n, d, K = w.n, w.d, w.K
    rng = np.random.default_rng(20220712)
    dims = [d] + LC_WIDTHS
    Ws_np = [(rng.normal(size=(dims[t], dims[t + 1])) / np.sqrt(dims[t])).astype(np.float32) for t in range(len(LC_WIDTHS))]
    Ws = [torch.from_numpy(W).cuda() for W in Ws_np]
    gamma = [0.1 * 0.9 ** k for k in range(K)] + [0.9 ** K]          # PPR-initialised hop weights
    perm_np = rng.permutation(n).astype(np.int32)
    perm = torch.from_numpy(perm_np).cuda()
    B = args.lc_batch if args.lc_batch > 0 else n
    batches = [perm[i:i + B] for i in range(0, n, B)] if B < n else [None]
    H = torch.empty((n, LC_WIDTHS[-1]), device="cuda")
    outs = [H[i:i + B] for i in range(0, n, B)] if B < n else [H]

    def step():
        for b, o in zip(batches, outs):
            gp.lc_forward_tensors(stack, b, gamma, Ws, out=o)

    for _ in range(max(args.warmup, 1)):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    ms_per_step = e0.elapsed_time(e1) / args.steps
    gp.gp_profile_enable(True)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    launches, mlp_ms = gp.gp_profile_read("gp_lc_mlp")
    _, red_ms = gp.gp_profile_read("gp_lc_reduce")
    gp.gp_profile_enable(False)
    flops_per_row = 2 * sum(dims[t] * dims[t + 1] for t in range(len(LC_WIDTHS))) * (K + 1)
    rows_per_launch = n / max(launches / args.steps, 1)
    avg_launch_s = mlp_ms * 1e-3 / max(launches, 1)
    achieved = rows_per_launch * flops_per_row / avg_launch_s / 1e12
    rec = {
        "metric": "LC-version forward rows/s over the K-hop stack",
        "value": round(n / (ms_per_step * 1e-3) / 1e6, 3), "unit": "Mrows/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": WORKLOAD_NAMES[args.workload] + "; consumer: GPRGNN_LC forward, widths "
                               + "-".join(map(str, dims)) + f", {K + 1} hops, batch {B}", "n": n, "d": d, "K": K,
                   "calls_per_step": len(batches)},
        "roofline": {"bound": "mfma", "achieved": round(achieved, 2), "peak": MFMA_F32_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(achieved / MFMA_F32_PEAK_TFLOPS, 4), "traffic": None, "kernel": "gp_lc_mlp",
                     "launches": launches, "avg_launch_us": round(avg_launch_s * 1e6, 3),
                     "algorithmic_flops_per_launch": int(rows_per_launch * flops_per_row)},
        "other_kernels_ms_per_step": {"gp_lc_reduce": round(red_ms / args.steps, 5)},
        "host_s": {"generate": round(t_gen, 2), "gp_plan_blocks": round(t_plan, 3)},
    }
    if cpu_baseline and not args.no_cpu_baseline:
        from oracle import lc
        stack_np = stack.cpu().numpy()
        rows, t_cpu = 0, 0.0
        i = 0
        while t_cpu < 10.0:                                # bounded sample: whole mini-batches, about 10 s
            ids = perm_np[i:i + 4096]
            t0 = time.perf_counter()
            lc.lc_forward(stack_np, ids, gamma, Ws_np)
            t_cpu += time.perf_counter() - t0
            rows += len(ids)
            i = (i + 4096) % max(n - 4096, 1)
        rec["cpu_baseline"] = {"value": round(rows / t_cpu / 1e6, 4), "unit": "Mrows/s", "cores": int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)),
                               "kind": "oracle", "sample": f"{rows} rows in mini-batches of 4096, fp64 numpy, {t_cpu:.2f} s"}
    return rec


def cpu_model() -> str:
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def time_workload(args, gp, torch, workload: int, cpu_baseline: bool):
    """Plans, times and (optionally) baselines one workload; returns its record, or an
    int return code when --lc took over."""
    import gp_synth
    dev = torch.device("cuda:0")
    t0 = time.time()
    w = gp_synth.make_workload(workload, scale=args.scale, contiguous_ids=args.contiguous_ids)
    memory = args.memory or ("pinned" if w.streamed else "device")
    t_gen = time.time() - t0
    budget = w.block_budget_edges
    if budget is None:
        budget = -(-gp_synth.stored_nonzeros_upper_bound(w.n, w.m, w.flags) // w.n_blocks)
    t0 = time.time()
    plan = gp.gp_plan_blocks(w.src, w.dst, w.n, budget, w.flags | (gp.GP_PLAN_ON_DEVICE if args.plan_on_device else 0))
    t_plan = time.time() - t0
    n, nnz, d, K = w.n, plan.nnz, w.d, w.K
    elem = 4 if w.dtype == gp.GP_F32 else 2
    tdt = torch.float32 if w.dtype == gp.GP_F32 else torch.bfloat16

    X = torch.from_numpy(w.X) if w.dtype == gp.GP_F32 else torch.from_numpy(w.X.view(np.int16)).view(torch.bfloat16)
    # The stack's leading dimension is the caller's: in HBM its rows start on 128-byte lines where that costs at
    # most 2 % more memory (d = 602: 608 elements), so that a gathered row touches no line it does not need.
    ld = d
    if memory == "device" and not args.lc:
        per_line = 128 // elem
        padded = -(-d // per_line) * per_line
        if (padded - d) * 50 <= d:
            ld = padded
    if memory == "device":
        X = X.to(dev)
        out = torch.empty((K + 1, n, ld), dtype=tdt, device=dev)
        stream = torch.cuda.current_stream().cuda_stream
    else:                                    # streamed schedule: the call returns when the stack is on the host
        X = X.pin_memory()
        out = torch.empty((K + 1, n, d), dtype=tdt).pin_memory()
        stream = None

    def step():
        gp.gp_propagate(plan, X.data_ptr(), d, d, w.dtype, w.agg, K, out.data_ptr(), ld, stream)

    if args.lc:
        if memory != "device":
            print("bench.py: --lc needs the stack in HBM (device memory)", file=sys.stderr)
            return 2
        step()
        torch.cuda.synchronize()
        args.workload = workload
        if args.lc == "both":           # the consumer rides along with the default run: all rows at once, and the paper's batch size
            recs = []
            for batch in (0, 4096):
                args.lc_batch = batch
                recs.append(bench_lc(args, gp, torch, w, plan, out, t_gen, t_plan, cpu_baseline=False))
            plan.close()
            return recs
        rec = bench_lc(args, gp, torch, w, plan, out, t_gen, t_plan)
        plan.close()
        print(json.dumps(rec))
        return 0

    t0 = time.perf_counter()
    step()                                   # the first call also uploads the plan and sizes the scratch
    torch.cuda.synchronize()
    t_first = time.perf_counter() - t0
    for _ in range(max(args.warmup, 1) - 1):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    # device operands: HIP events on the launch stream; pinned operands: the call is
    # synchronous and works on its own streams, so the host clock is the measure
    ms_per_step = e0.elapsed_time(e1) / args.steps if memory == "device" else wall * 1e3 / args.steps
    efu = nnz * d * K
    value = efu / (ms_per_step * 1e-3) / 1e9

    # a second, untimed pass brackets every step with its own event pair: median and minimum
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    per_step = []
    for i in range(args.steps):
        if memory == "device":
            marks[i].record()
        t0 = time.perf_counter()
        step()
        per_step.append((time.perf_counter() - t0) * 1e3)
    if memory == "device":
        marks[args.steps].record()
    torch.cuda.synchronize()
    if memory == "device":
        per_step = [marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps)]

    # dominant kernel: per-launch duration from HIP events the library records around each
    # launch on the launch stream.  The event pairs themselves cost time between the
    # launches, so this pass runs a few per cent slower than the timed one (its own
    # ms per step is reported beside the kernel times); the durations are the kernels' own.
    gp.gp_profile_enable(True)
    b0, b1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    b0.record()
    for _ in range(args.steps):
        step()
    b1.record()
    torch.cuda.synchronize()
    bracketed_ms = b0.elapsed_time(b1) / args.steps if memory == "device" else (time.perf_counter() - t0) * 1e3 / args.steps
    # a hop is one launch of the segment kernel, or several where the plan's cache schedule cuts every segment
    # into the non-zeros whose source row can be kept close and the others (the former then go through a second
    # launch of the segment kernel, or through the LDS kernel, which for shared lists has a packing launch before
    # it); the roofline figures below are per launch, the mean over all of a hop's launches
    seg_launches, seg_ms = gp.gp_profile_read("gp_hop_segments")
    lds_launches, lds_ms = gp.gp_profile_read("gp_hop_cluster_lds")
    pack_launches, pack_ms = gp.gp_profile_read("gp_pack_strips")
    launches, hop_ms = seg_launches + lds_launches + pack_launches, seg_ms + lds_ms + pack_ms
    fix_launches, fix_ms = gp.gp_profile_read("gp_fixup_rows")
    _, copy_ms = gp.gp_profile_read("gp_copy_rows")
    gp.gp_profile_enable(False)
    avg_launch_s = hop_ms * 1e-3 / max(launches, 1)
    # one launch covers a whole hop on device operands; the streamed schedule launches
    # once per edge block and column slab, each launch doing its share of the hop
    launches_per_hop = max(1, round(launches / max(args.steps * K, 1)))
    bytes_per_launch = algorithmic_bytes_per_hop(n, nnz, d, elem) // launches_per_hop
    achieved = bytes_per_launch / avg_launch_s / 1e9
    options = {k: gp.gp_get_option(k) for k in ("segment_edges", "column_tile", "column_slices", "cache_schedule", "split_records", "lds_pass", "hub_pass")}
    recorded = recorded_traffic(workload, options) if (args.scale == 1.0 and memory == "device" and not args.contiguous_ids) else None
    traffic = recorded.get("bytes_per_launch") if recorded else None

    def kernel_record(name, count, ms):
        # launches and mean duration of one of the hop's kernels in this run; with the recorded counters, the bytes
        # one launch of it moved (fetch + write) and the rate that makes against the HBM peak
        out = {"launches": count, "avg_launch_us": round(ms * 1e3 / max(count, 1), 3)}
        moved = (recorded or {}).get("per_kernel", {}).get(name)
        if moved and count:
            b = moved["fetch_bytes"] + moved["write_bytes"]
            out["traffic"] = b
            out["traffic_frac"] = round(b / (ms * 1e-3 / count) / 1e9 / HBM_PEAK_GBS, 4)
        return out
    flops_per_launch = 2 * nnz * d // launches_per_hop          # one multiply-add per non-zero and column
    gathered_per_launch = nnz * d * elem // launches_per_hop    # bytes the lanes read if every row comes from cache
    S, slice_elems, _, _ = plan.work_lists(d, w.dtype, max(1, min(16 // elem, d)))
    sched = None
    if lds_launches:
        sched = plan.lds_schedule(0, d)
        kind = {1: "in-cluster non-zeros", 2: "non-zeros whose source is one of the 10192 most popular rows"}[sched["hot_mode"]]
        work_lists = (f"{kind} from LDS (strips of 4 columns, {sched['ids'].size} reads for {int((sched['rest']['slice'] != 0).sum())} "
                      f"segments, {'conflict-free' if sched['conflict_free'] else 'column-list'} order), the others as implicit lists")
    elif S:
        work_lists = "explicit per XCD, %d column slices of %d" % (S, slice_elems)
    else:
        work_lists = "implicit"
    hop_kernel = "gp_hop_segments" + (" + gp_hop_cluster_lds" if lds_launches else "") + (" + gp_pack_strips" if pack_launches else "")

    rec = {
        "metric": "edge-feature updates/s (GEFU/s) for K-hop A^k X precompute",
        "value": round(value, 3),
        "unit": "GEFU/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "ms_per_step_median": round(float(np.median(per_step)), 5),
        "ms_per_step_min": round(float(np.min(per_step)), 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32" if w.dtype == gp.GP_F32 else "bf16 storage, f32 accumulate",
        "data": "synthetic",
        "config": {"workload": WORKLOAD_NAMES[workload] + (" [community-contiguous ids]" if args.contiguous_ids else "")
                   + (f" [scale {args.scale}]" if args.scale != 1.0 else ""), "memory": memory, "n": n, "nnz": nnz, "d": d, "stack_ld": ld, "K": K,
                   "edge_blocks": plan.num_blocks, "agg": ["sym", "mean", "sum"][w.agg],
                   "segments": int(plan.segments.size), "partial_rows": plan.num_partial_rows,
                   "work_lists": work_lists,
                   "options": options},
        "roofline": {"bound": "hbm", "achieved": round(achieved, 2), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                     # the same launch on the bytes the counters saw (fetch + write, per launch): how busy the memory system was
                     "traffic_frac": round(traffic / avg_launch_s / 1e9 / HBM_PEAK_GBS, 4) if traffic else None,
                     "kernel": hop_kernel, "launches": launches, "launches_per_hop": launches_per_hop,
                     "per_kernel": {"gp_hop_segments": kernel_record("gp_hop_segments", seg_launches, seg_ms),
                                    "gp_hop_cluster_lds": kernel_record("gp_hop_cluster_lds", lds_launches, lds_ms),
                                    "gp_pack_strips": kernel_record("gp_pack_strips", pack_launches, pack_ms)},
                     "avg_launch_us": round(avg_launch_s * 1e6, 3), "algorithmic_bytes_per_launch": bytes_per_launch,
                     "kernel_times_from": f"event-bracketed pass, {bracketed_ms:.5f} ms per step",
                     # the other ceilings of the same launch: plain fp32 vector arithmetic, and the rate at
                     # which the lanes are fed gathered rows (useful bytes only)
                     "other_bounds": {
                         "alu": {"achieved": round(flops_per_launch / avg_launch_s / 1e12, 3), "peak": FP32_VECTOR_PEAK_TFLOPS,
                                 "unit": "TFLOP/s", "frac": round(flops_per_launch / avg_launch_s / 1e12 / FP32_VECTOR_PEAK_TFLOPS, 4)},
                         "gathered_rows": {"achieved": round(gathered_per_launch / avg_launch_s / 1e9, 1), "unit": "GB/s",
                                           "note": "nnz * d * element size per launch over its duration; rows served by the "
                                                   "XCDs' L2 arrive at 20 - 27 TB/s on this machine, rows that miss it at about 7"}}},
        # the launch that serves the hot non-zeros from LDS: reads of 16 bytes (padding included) over its own duration
        "lds_launch": None if not sched else {
            "bound": "lds", "unit": "GB/s", "peak": LDS_PEAK_GBS,
            "achieved": round(int(sched["ids"].size) * ((d + 3) // 4) * 16 / (lds_ms * 1e-3 / lds_launches) / 1e9, 1),
            "frac": round(int(sched["ids"].size) * ((d + 3) // 4) * 16 / (lds_ms * 1e-3 / lds_launches) / 1e9 / LDS_PEAK_GBS, 4),
            "reads_per_strip": int(sched["ids"].size), "strips": (d + 3) // 4, "avg_launch_us": round(lds_ms * 1e3 / lds_launches, 3),
            "note": "random 16-byte reads come out of LDS at 52 - 57 TB/s on this machine, conflict-free ones (this schedule's) at "
                    "about 100 with the index arithmetic of a read, sequential ones at 146; 5.6 vector instructions per read allow 112"},
        "other_kernels_ms_per_step": {"gp_fixup_rows": round(fix_ms / args.steps, 5),
                                      "gp_copy_rows": round(copy_ms / args.steps, 5)},
        "host_s": {"generate": round(t_gen, 2), "gp_plan_blocks": round(t_plan, 3), "planned_on": "gpu" if args.plan_on_device else "host",
                   "first_call_with_plan_upload": round(t_first, 4), "timed_wall": round(wall, 3)},
    }

    if memory == "pinned":
        # bytes that must cross the host link per step: X in, K hop slabs out (slab 0 = X is a
        # host-side copy), every edge block at least once (again per hop and column slab
        # when the HBM budget cannot keep them)
        slabs = max(1, launches // max(args.steps * K * plan.num_blocks, 1))
        link_bytes = n * d * elem * (K + 1) + 4 * nnz + 16 * int(plan.segments.size)
        rec["host_link"] = {"min_bytes_per_step": link_bytes, "GB/s_on_min_bytes": round(link_bytes / (ms_per_step * 1e-3) / 1e9, 2),
                            "column_slabs": slabs}
    if cpu_baseline:
        import oracle
        cores = min(16, os.cpu_count() or 1)
        del out
        op = oracle.plan_blocks(w.src, w.dst, n, budget, w.flags)
        Xw = (w.X if w.dtype == gp.GP_F32 else gp_synth.bf16_bits_to_f32(w.X)).astype(np.float64)
        # bounded sample: whole hops of the same workload (the K-hop chain restarted
        # from X when it ends) until about 10 s of CPU work have been timed
        hops, t_cpu = 0, 0.0
        cur = Xw
        while t_cpu < 10.0:
            t0 = time.perf_counter()
            cur = oracle.hop(op, cur, w.agg, threads=cores)
            t_cpu += time.perf_counter() - t0
            hops += 1
            if hops % K == 0:
                cur = Xw
        rec["cpu_baseline"] = {"value": round(nnz * d * hops / t_cpu / 1e9, 4), "unit": "GEFU/s", "cores": cores,
                               "kind": "oracle", "sample": f"{hops} hops ({hops / K:.1f} passes of the K={K} chain) of "
                                                            f"the same workload, fp64, {t_cpu:.2f} s",
                               "cpu": cpu_model()}
        if t_cpu / hops * cores < 3.0:
            # the same loop on one thread, a shorter sample (about 3 s), where a hop is short enough
            hops1, t1 = 0, 0.0
            cur = Xw
            while t1 < 3.0:
                t0 = time.perf_counter()
                cur = oracle.hop(op, cur, w.agg, threads=1)
                t1 += time.perf_counter() - t0
                hops1 += 1
                if hops1 % K == 0:
                    cur = Xw
            rec["cpu_baseline"]["single_thread_value"] = round(nnz * d * hops1 / t1 / 1e9, 4)
    plan.close()
    return rec


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="all",
                    help="all (default): the four workloads that are resident in HBM, the line being the largest one's; "
                         "or one of 1..5")
    ap.add_argument("--scale", type=float, default=1.0,
                    help="shrink node and pair counts together (workload 5 is only practical below 1)")
    ap.add_argument("--memory", choices=["device", "pinned"], default=None,
                    help="where X and the stack live: device (resident schedule) or pinned host memory "
                         "(streamed schedule; the default for workload 5)")
    ap.add_argument("--hbm-budget-gb", type=float, default=0.0, help="streamed schedule: HBM budget (0 = automatic)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--option", action="append", default=[], metavar="NAME=VALUE",
                    help="library option (gp_set_option), e.g. column_tile=32")
    ap.add_argument("--lc", action="store_true",
                    help="time the LC-version forward pass (gp_lc_forward) over the hop stack instead of the precompute")
    ap.add_argument("--lc-batch", type=int, default=4096, help="--lc: mini-batch rows per call (0 = all rows in one call)")
    ap.add_argument("--plan-on-device", action="store_true",
                    help="gp_plan_blocks with GP_PLAN_ON_DEVICE: the non-zero set sorted and de-duplicated on the GPU "
                         "(the plan is the same; host_s.gp_plan_blocks shows the time)")
    ap.add_argument("--contiguous-ids", action="store_true",
                    help="workload 4 only: community-contiguous node ids (locality given) instead of permuted ids")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus must be 1 (no multi-GPU path exists)", file=sys.stderr)
        return 2
    if args.workload != "all" and args.workload not in [str(k) for k in WORKLOAD_NAMES]:
        print("bench.py: --workload must be all or 1..5", file=sys.stderr)
        return 2

    import torch
    import paper_2207_12000_amd as gp
    if not os.path.exists(gp.LIB_PATH):      # load what is built; build only if nothing is
        from paper_2207_12000_amd import build as libbuild
        libbuild.build()

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(torch.device("cuda:0"))

    for kv in args.option:
        name, val = kv.split("=")
        gp.gp_set_option(name, int(val))
    if args.hbm_budget_gb > 0:
        gp.gp_set_hbm_budget_bytes(int(args.hbm_budget_gb * 2**30))

    if args.workload != "all":
        rec = time_workload(args, gp, torch, int(args.workload), not args.no_cpu_baseline)
        if isinstance(rec, int):
            return rec
        print(json.dumps(rec))
        return 0
    if args.lc:
        rc = time_workload(args, gp, torch, 2, False)
        return rc if isinstance(rc, int) else 0

    # every in-HBM workload; the line is the largest one's, the others ride along in short form
    others = {}
    head = None
    for wl in IN_HBM_WORKLOADS:
        rec = time_workload(args, gp, torch, wl, wl == HEADLINE_WORKLOAD and not args.no_cpu_baseline)
        torch.cuda.empty_cache()
        if wl == HEADLINE_WORKLOAD:
            head = rec
        else:
            others[f"config{wl}"] = {
                "workload": rec["config"]["workload"], "value": rec["value"], "unit": rec["unit"],
                "ms_per_step": rec["ms_per_step"], "work_lists": rec["config"]["work_lists"],
                "roofline": {k: rec["roofline"][k] for k in ("bound", "achieved", "peak", "unit", "frac", "traffic", "traffic_frac",
                                                             "avg_launch_us", "algorithmic_bytes_per_launch")},
                "host_s": rec["host_s"]}
    head["other_workloads"] = others
    # the LC-version consumer over config 2's stack (its own metric and roofline: fp32 MFMA), in short form
    args.lc = "both"
    lc_recs = time_workload(args, gp, torch, 2, False)
    if isinstance(lc_recs, list):
        head["lc_consumer"] = [{"workload": r["config"]["workload"], "value": r["value"], "unit": r["unit"],
                                "ms_per_step": r["ms_per_step"],
                                "roofline": {k: r["roofline"][k] for k in ("bound", "achieved", "peak", "unit", "frac", "avg_launch_us")}}
                               for r in lc_recs]
    print(json.dumps(head))
    return 0


if __name__ == "__main__":
    sys.exit(main())
