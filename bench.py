#!/usr/bin/env python3
"""Benchmark of the schedule executor on one MI355X.

A step is one sccl_execute of the whole schedule (all S steps of sends) on P virtual ranks'
buffers resident in HBM.  Default workload: Allreduce fp32, 8 ranks x 256 MiB on the 8-node
graph (configuration 3).  Every step is timed with HIP events recorded on the stream the kernel
is launched on; the in-place buffers are restored from a pristine device copy between steps,
outside the timed windows.

Prints ONE JSON line on stdout.  `--report FILE` additionally times the other configurations and
writes a markdown table to FILE.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth

# Bytes that left the L2 per launch, from two rocprofv3 --pmc runs (FETCH_SIZE, then WRITE_SIZE), each scaled by
# what the same counter reads for the 1 GiB copy kernel (FETCH_SIZE x 2.000, WRITE_SIZE x 1.000).  Keyed by
# (workload, grid, block_threads, vectors_per_thread); the figures and commands are in profiles/.
MEASURED_TRAFFIC = {
    ("cfg3", 256, 256, 4): (2 * 1097471.0 + 2658935.8) * 1024,
    ("cfg4", 256, 256, 8): (2 * 2542746.1 + 7158514.2) * 1024,
    ("cfg2", 256, 256, 8): (2 * 124550.7 + 458752.0) * 1024,
}


def make_inputs(wl, sf, device):
    """Pristine device buffers for a workload (seeded, generated on the device; bit-identical to the host recipe
    for the integer-derived distributions)."""
    import torch
    from paper_2008_08708_amd import inputs
    n_elems = wl.bytes_per_rank // wl.elem_bytes
    epc = n_elems // sf.positions_per_rank
    bufs = []
    for n in range(sf.num_nodes):
        b = inputs.torch_rank_buffer(wl.dist, wl.dtype, wl.seed, n, n_elems, device)
        if wl.poison_non_owned:
            view = b.view(torch.int32 if wl.elem_bytes == 4 else torch.int16)
            pat = inputs.POISON_U32 if wl.elem_bytes == 4 else inputs.POISON_U16
            held = {int(c if sf.slot is None else sf.slot[c, n]) for c in range(sf.num_chunks) if sf.pre[c, n]}
            for k in range(sf.positions_per_rank):
                if k not in held:
                    view[k * epc:(k + 1) * epc] = pat
        bufs.append(b)
    return bufs, epc


def time_workload(wl, steps, warmup, options=None, keep=False, mode="sccl_execute"):
    """Returns dict with per-step kernel times (ms) measured by events on the launch stream."""
    import torch
    from paper_2008_08708_amd import schedule_file, sccl
    dev = torch.device("cuda:0")
    sf = schedule_file.load(wl.schedule)
    pristine, epc = make_inputs(wl, sf, dev)
    work = [torch.empty_like(b) for b in pristine]
    plan = sccl.sccl_plan_create(*sf.descriptions(wl.dtype, epc), options=options)
    stats = sccl.sccl_plan_stats(plan)
    stream = torch.cuda.current_stream()
    execute = getattr(sccl, mode)

    def restore():
        for w, p in zip(work, pristine):
            w.copy_(p)

    for _ in range(warmup):
        restore()
        execute(plan, work, stream)
    torch.cuda.synchronize()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for a, b in evs:
        restore()                      # outside the timed window
        a.record(stream)
        execute(plan, work, stream)
        b.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms = [a.elapsed_time(b) for a, b in evs]
    out = {"ms": ms, "wall_s": wall, "stats": stats, "sf": sf, "epc": epc}
    if keep:
        out.update({"pristine": pristine, "work": work, "plan": plan})
    else:
        sccl.sccl_plan_destroy(plan)
    return out


def graph_us_per_execute(wl, count=20, reps=10, options=None):
    """Microseconds per sccl_execute when `count` of them run back to back inside one HIP graph (values are not
    restored in between: only the time is of interest).  This is what a launch-bound caller pays per collective."""
    import torch
    from paper_2008_08708_amd import schedule_file, sccl
    sf = schedule_file.load(wl.schedule)
    work, epc = make_inputs(wl, sf, torch.device("cuda:0"))
    plan = sccl.sccl_plan_create(*sf.descriptions(wl.dtype, epc), options=options)
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        for _ in range(count):
            sccl.sccl_execute(plan, work, side)
    times = []
    for _ in range(reps + 2):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        graph.replay()
        b.record()
        torch.cuda.synchronize()
        times.append(a.elapsed_time(b) * 1e3 / count)
    del graph
    sccl.sccl_plan_destroy(plan)
    times = sorted(times[2:])
    return times[len(times) // 2]


def copy_ceiling(nbytes, reps=10):
    """GB/s (read + write) of a plain 16-byte-per-lane copy kernel over nbytes."""
    import torch
    from paper_2008_08708_amd import sccl
    src = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0").random_(0, 255)
    dst = torch.empty_like(src)
    stream = torch.cuda.current_stream()
    for _ in range(2):
        sccl.sccl_copy_kernel(dst, src, nbytes, stream)
    evs = []
    for _ in range(reps):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(stream)
        sccl.sccl_copy_kernel(dst, src, nbytes, stream)
        b.record(stream)
        evs.append((a, b))
    torch.cuda.synchronize()
    ms = sorted(a.elapsed_time(b) for a, b in evs)
    return 2.0 * nbytes / (ms[len(ms) // 2] * 1e-3) / 1e9


def cpu_baseline(run, wl):
    """The oracle, as it stands, on the host cores: the full workload, same plan, same input bits.
    Also compares the GPU's result with it, bit for bit, on the full buffers."""
    import numpy as np
    import torch
    from oracle import executor, schedule as osched
    from paper_2008_08708_amd import sccl
    sf, epc = run["sf"], run["epc"]
    sched = osched.Schedule(sf.rounds, sf.sends)
    threads = min(16, os.cpu_count() or 1, executor.max_threads())
    layout = {} if sf.slot is None else {"slot": sf.slot, "slots_per_rank": sf.slots_per_rank}
    host_in = [p.cpu().numpy() for p in run["pristine"]]
    times = []
    host = None
    for rep in range(3):
        host = [h.copy() for h in host_in]
        t0 = time.perf_counter()
        executor.execute(wl.dtype, sf.num_chunks, epc, sched, host, threads=threads, **layout)
        times.append(time.perf_counter() - t0)
    # the GPU's result on the same inputs
    for w, p in zip(run["work"], run["pristine"]):
        w.copy_(p)
    sccl.sccl_execute(run["plan"], run["work"])
    torch.cuda.synchronize()
    same = True
    for n, w in enumerate(run["work"]):
        g = w.cpu().numpy()
        u = np.uint32 if g.dtype.itemsize == 4 else np.uint16
        if not (g.view(u) == host[n].view(u)).all():
            same = False
    med = sorted(times)[1]
    host1 = [h.copy() for h in host_in]
    t0 = time.perf_counter()
    executor.execute(wl.dtype, sf.num_chunks, epc, sched, host1, threads=1, **layout)
    one = time.perf_counter() - t0
    return {"value": run["stats"]["bytes_min"] / med / 1e9, "unit": "GB/s", "cores": threads, "kind": "oracle",
            "value_one_core": run["stats"]["bytes_min"] / one / 1e9,
            "sample": f"the full workload ({run['stats']['bytes_min'] / 2**30:.2f} GiB algorithmic), median of 3 runs, "
                      f"OpenMP over the element range"}, same


def sweep(wl, steps, warmup):
    """Every launch shape of the through-memory kernel (workgroup size x vectors per lane x workgroups per CU) and,
    where the cells fit, of the staged kernel (slice x workgroup size); one JSON line each, the best last."""
    from paper_2008_08708_amd import sccl
    shapes = [{"lowering": 1, "block_threads": bt, "vectors_per_thread": vt, "max_workgroups": 256 * k}
              for bt in (64, 128, 256) for vt in (1, 2, 4, 8) for k in (1, 2, 4)]
    shapes += [{"lowering": 2, "slice_vectors": sv, "staged_threads": th}
               for sv in (1, 2, 4, 8, 16, 32, 64, 128) for th in (256, 512, 1024)]
    best = None
    for o in shapes:
        try:
            r = time_workload(wl, steps, warmup, o)
        except sccl.ScclError:
            continue                                   # a staged shape whose cells do not fit
        ms = sorted(r["ms"])
        st = r["stats"]
        rec = {"workload": wl.name, "options": o, "grid": st["grid_workgroups"], "median_us": round(ms[len(ms) // 2] * 1e3, 2),
               "min_us": round(ms[0] * 1e3, 2), "effective_GBs": round(st["bytes_min"] / ms[len(ms) // 2] / 1e6, 1)}
        print(json.dumps(rec), flush=True)
        if best is None or rec["median_us"] < best["median_us"]:
            best = rec
    print(json.dumps({"best": best}), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg3")
    ap.add_argument("--block-threads", type=int, default=0)
    ap.add_argument("--vectors-per-thread", type=int, default=0)
    ap.add_argument("--max-workgroups", type=int, default=0)
    ap.add_argument("--lowering", type=int, default=0, help="0 = the plan chooses, 1 = through memory, 2 = staged in the local data share")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--report", default="", metavar="FILE", help="also time the other configurations; markdown table to FILE")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the benchmark line: time --workload under every launch shape of both kernels "
                         "(the paper's search over thread-block count and size, section 4) and print one JSON line each")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build executes P virtual ranks on ONE GPU; --gpus N with N > 1 is not supported "
              "(no inter-GPU path exists in this repository)", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2008_08708_amd import sccl, workloads
    sccl.lib()                                    # fails loudly when the HIP library is not built
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    options = {k: v for k, v in (("block_threads", args.block_threads), ("vectors_per_thread", args.vectors_per_thread),
                                 ("max_workgroups", args.max_workgroups), ("lowering", args.lowering)) if v}
    if args.workload.startswith("cfg5:"):             # cfg5:<allgather|allreduce>:<bytes per rank>
        _, coll_name, size = args.workload.split(":")
        wl = workloads.sweep_workload(coll_name, int(size))
    else:
        wl = workloads.WORKLOADS[args.workload]
    if args.sweep:
        sweep(wl, args.steps, args.warmup)
        return
    run = time_workload(wl, args.steps, args.warmup, options or None, keep=True)
    st = run["stats"]
    ms = run["ms"]
    mean_ms = sum(ms) / len(ms)
    gbs = st["bytes_min"] / (mean_ms * 1e-3) / 1e9
    line = {
        "metric": "effective HBM GB/s (% peak) executing Allreduce, 8 ranks x 256 MiB fp32"
                  if args.workload == "cfg3" else f"effective HBM GB/s executing {wl.schedule}",
        "value": round(gbs, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(mean_ms, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": {"f32": "f32", "f16": "f16 (f32 accumulate)", "i32": "i32"}[wl.dtype], "data": "synthetic",
        "config": {"workload": f"{wl.name}: {wl.schedule}, P={st['num_nodes']} virtual ranks x "
                               f"{wl.bytes_per_rank >> 20} MiB {wl.dtype}, G={st['num_global_chunks']} chunks, "
                               f"S={st['num_steps']} steps, {st['num_sends']} sends",
                   "bytes_min": st["bytes_min"], "bytes_unfused": st["bytes_unfused"],
                   "grid": st["grid_workgroups"], "block_threads": st["block_threads"],
                   "vectors_per_thread": st["vectors_per_thread"]},
        "pct_of_hbm_peak": round(100.0 * gbs / HBM_PEAK_GBS, 2),
        "ms_min": round(min(ms), 4), "ms_median": round(sorted(ms)[len(ms) // 2], 4),
        "wall_ms_per_step_incl_restore": round(run["wall_s"] * 1e3 / args.steps, 4),
        "roofline": {"bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(gbs / HBM_PEAK_GBS, 4),
                     "traffic": MEASURED_TRAFFIC.get((args.workload, st["grid_workgroups"], st["block_threads"],
                                                      st["vectors_per_thread"])),
                     "kernel": ("sccl_staged_kernel" if st["lowering"] == 2 else "sccl_exec_kernel") + " (one launch = the whole schedule)",
                     "algorithmic_bytes_per_launch": st["bytes_min"]},
    }
    try:
        line["copy_kernel_ceiling_gbs"] = round(copy_ceiling(1 << 30), 1)
    except Exception as e:                        # measurement aid only
        line["copy_kernel_ceiling_gbs"] = None
        print(f"copy ceiling failed: {e}", file=sys.stderr)
    if not args.no_cpu_baseline:
        base, same = cpu_baseline(run, wl)
        line["cpu_baseline"] = base
        line["parity_full_buffers_bitwise"] = bool(same)
    sccl.sccl_plan_destroy(run["plan"])
    del run
    torch.cuda.empty_cache()

    if args.report:
        rows = []
        names = [("cfg1", workloads.WORKLOADS["cfg1"]), ("cfg2", workloads.WORKLOADS["cfg2"]),
                 ("cfg3", workloads.WORKLOADS["cfg3"]), ("cfg4", workloads.WORKLOADS["cfg4"]),
                 ("cfg4b", workloads.WORKLOADS["cfg4b"])]
        names += [(k, workloads.WORKLOADS[k]) for k in ("alltoall", "broadcast", "reduce", "gather", "scatter")]
        for coll in ("allgather", "allreduce"):
            for size in workloads.sweep_sizes():
                names.append((f"cfg5 {coll} {size}", workloads.sweep_workload(coll, size)))
        from paper_2008_08708_amd.sccl import SCCL_LOWER_MEMORY, SCCL_LOWER_STAGED, ScclError

        def median_us(w, steps, mode, opts=None):
            r = time_workload(w, steps, 3, options=opts, mode=mode)
            m = sorted(r["ms"])
            out = (m[len(m) // 2] * 1e3, m[0] * 1e3, r["stats"])
            del r
            torch.cuda.empty_cache()
            return out

        for label, w in names:
            steps = 5 if w.bytes_per_rank >= (1 << 30) else 20
            med, mn, s = median_us(w, steps, "sccl_execute")                     # the default: lowering chosen by the plan
            mem_med = med if s["lowering"] == SCCL_LOWER_MEMORY else median_us(w, steps, "sccl_execute", {"lowering": SCCL_LOWER_MEMORY})[0]
            stg_med = None
            if s["lowering"] == SCCL_LOWER_STAGED:
                stg_med = med
            elif s["staged_available"] and w.bytes_per_rank <= (16 << 20):
                try:
                    stg_med = median_us(w, steps, "sccl_execute", {"lowering": SCCL_LOWER_STAGED})[0]
                except ScclError:
                    stg_med = None
            graph_us = graph_us_per_execute(w) if w.bytes_per_rank <= (1 << 20) else None
            oracle = None                                    # (GB/s on the host cores, GB/s on one core, cores, bitwise equal)
            if s["num_nodes"] * w.bytes_per_rank <= (4 << 30):
                kept = time_workload(w, 1, 0, keep=True)
                base, same = cpu_baseline(kept, w)
                oracle = (base["value"], base["value_one_core"], base["cores"], same)
                sccl.sccl_plan_destroy(kept["plan"])
                del kept
                torch.cuda.empty_cache()
            step_med, _, _ = median_us(w, steps, "sccl_execute_stepwise")
            cpy_med = median_us(w, steps, "sccl_execute_memcpy")[0] if s["num_reduce_groups"] == 0 else None
            rows.append((label, s["num_nodes"], w.bytes_per_rank, s["chunk_bytes"], s["num_steps"], s["bytes_min"],
                         med, mn, s["bytes_min"] / (med * 1e-6) / 1e9, "staged" if s["lowering"] == SCCL_LOWER_STAGED else "memory",
                         s["num_levels"], s["grid_workgroups"], mem_med, stg_med, step_med, cpy_med, graph_us, oracle))
            fmt = lambda x: "-" if x is None else format(x, ".1f")
            print(f"[report] {label}: default ({rows[-1][9]}) {med:.1f} us ({rows[-1][8]:.1f} GB/s), through memory {fmt(mem_med)} us, "
                  f"staged {fmt(stg_med)} us, per-step kernels {fmt(step_med)} us, per-send copies {fmt(cpy_med)} us, "
                  f"in a graph of 20 {fmt(graph_us)} us each",
                  file=sys.stderr, flush=True)
        os.makedirs(os.path.dirname(os.path.abspath(args.report)), exist_ok=True)
        with open(args.report, "w") as f:
            f.write("| workload | P | bytes/rank | chunk bytes | S | bytes_min | sccl_execute: median us | min us | effective GB/s | % of 8 TB/s "
                    "| lowering | levels | grid | through memory: us | staged: us | one kernel per step: us | one copy per send: us "
                    "| each of 20 in one HIP graph: us | oracle on the host cores: GB/s (cores) | oracle on one core: GB/s "
                    "| full buffers bitwise equal to the oracle's |\n")
            f.write("|" + "---|" * 21 + "\n")
            fmt = lambda x: "-" if x is None else format(x, ".1f")
            for r in rows:
                f.write(f"| {r[0]} | {r[1]} | {r[2]} | {r[3]} | {r[4]} | {r[5]} | {r[6]:.1f} | {r[7]:.1f} | {r[8]:.1f} | "
                        f"{100 * r[8] / HBM_PEAK_GBS:.1f} | {r[9]} | {r[10]} | {r[11]} | {fmt(r[12])} | {fmt(r[13])} | "
                        f"{fmt(r[14])} | {fmt(r[15])} | {fmt(r[16])} | "
                        + ("- | - | (sampled windows: tests/test_gpu_fullsize.py) |\n" if r[17] is None else
                           f"{r[17][0]:.1f} ({r[17][2]}) | {r[17][1]:.1f} | {'yes' if r[17][3] else 'NO'} |\n"))
        # ---- the paper's size-dependent choice between two algorithms (section 5.5) on this hardware: the
        # latency-optimal and the bandwidth-optimal torus algorithm at every size, the (alpha, beta) of the cost
        # model fitted to the measurements, and what the model would have chosen.
        with open(args.report, "a") as f:
            f.write("\n| collective | bytes/rank | latency-optimal: us | bandwidth-optimal: us | measured best | model's choice "
                    "| model us (latency / bandwidth) |\n|---|---|---|---|---|---|---|\n")
            for coll in ("allgather", "allreduce"):
                meas = []
                for size in workloads.sweep_sizes():
                    pair = []
                    for alg in ("latency", "bandwidth"):
                        w = workloads.sweep_workload(coll, size, alg)
                        steps = 5 if size >= (1 << 30) else 20
                        med, _, st_ = median_us(w, steps, "sccl_execute")
                        # the model's two coordinates: a = S, b = (R / C) * L = R * chunk bytes
                        pair.append((med * 1e-6, float(st_["num_steps"]), float(st_["num_rounds"]) * st_["chunk_bytes"]))
                    meas.append((size, pair))
                a = [p[1] for _, pair in meas for p in pair]
                b = [p[2] for _, pair in meas for p in pair]
                t = [p[0] for _, pair in meas for p in pair]
                alpha, beta = sccl.sccl_cost_fit(a, b, t)
                for size, pair in meas:
                    model = [p[1] * alpha + p[2] * beta for p in pair]
                    f.write(f"| {coll} | {size} | {pair[0][0] * 1e6:.1f} | {pair[1][0] * 1e6:.1f} | "
                            f"{'latency' if pair[0][0] <= pair[1][0] else 'bandwidth'} | "
                            f"{'latency' if model[0] <= model[1] else 'bandwidth'} | {model[0] * 1e6:.1f} / {model[1] * 1e6:.1f} |\n")
                f.write(f"\n{coll}: fitted alpha = {alpha * 1e6:.3f} us per step, beta = {beta * 1e12:.4f} ps per byte "
                        f"(1 / beta = {1e-9 / beta if beta > 0 else float('inf'):.0f} GB/s per link-equivalent)\n")
                print(f"[report] {coll}: alpha {alpha * 1e6:.3f} us, beta {beta * 1e12:.4f} ps/B", file=sys.stderr, flush=True)
        with open(args.report, "a") as f:
            f.write("\nContext, not a target: the paper gives no absolute time or bandwidth for executing a schedule in its "
                    "text, only speedups measured across eight GPUs over their links (section 5.5): Allgather up to 2.2x "
                    "(small) and 1.14x (large) over NCCL 2.7.8, Allreduce up to 1.8x (small, the 8-chunk algorithm) and 1.06x "
                    "(large, the 48-chunk algorithm), Alltoall more than 6.8x (large) over point-to-point copies, on a DGX-1 "
                    "(8 x V100, six 25 GB/s NVLink ports per GPU); Allgather faster than RCCL only at large sizes on a Gigabyte "
                    "Z52 (8 x MI50, xGMI about 33 GB/s, PCIe 4 about 27 GB/s).  Nothing here reproduces an inter-GPU link: the "
                    "figures above are one MI355X moving P virtual ranks' buffers inside its own HBM "
                    f"(peak {HBM_PEAK_GBS / 1000:.0f} TB/s).\n")
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
