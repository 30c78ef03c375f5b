#!/usr/bin/env python3
"""Benchmark of the schedule executor on one MI355X.

A step is one sccl_execute of the whole schedule (all S steps of sends) on P virtual ranks'
buffers resident in HBM.  Default workload: Allreduce fp32, 8 ranks x 256 MiB on the 8-node
graph (configuration 3).  Every step is timed with HIP events recorded on the stream the kernel
is launched on; the in-place buffers are restored from a pristine device copy between steps,
outside the timed windows.

Prints ONE JSON line on stdout.  `--report FILE` additionally times the other configurations and
writes a markdown table to FILE; `--ceilings` prints what plain streaming kernels reach on this GPU.
"""
import argparse
import ctypes
import glob
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
LOWERING_NAMES = {1: "memory", 2: "staged"}


# ---- measurement aids: plain streaming kernels of known traffic (bench_kernels.hip, not part of the library)

_aid = None


def bench_kernels():
    global _aid
    if _aid is None:
        path = os.path.join(ROOT, "libbench_kernels.so")
        if not os.path.exists(path):                          # nothing built yet: build once, in-tree
            from paper_2008_08708_amd import build as _build
            _build.build_bench_kernels()
        import torch  # noqa: F401  (one HIP runtime per process: torch's, loaded first)
        L = ctypes.CDLL(path)
        L.bench_stream.restype = ctypes.c_int
        L.bench_stream.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int,
                                   ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
        L.bench_empty.restype = ctypes.c_int
        L.bench_empty.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
        _aid = L
    return _aid


def launch_floor_us(grid=256, threads=64, reps=30):
    """Median microseconds between two HIP events around a kernel that does nothing: what any single launch costs
    on this machine before its work starts (the floor under every small-size figure)."""
    import torch
    sink = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    s = torch.cuda.current_stream().cuda_stream
    times = []
    for r in range(reps + 3):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        if bench_kernels().bench_empty(grid, threads, ctypes.c_void_p(sink.data_ptr()), ctypes.c_void_p(int(s))) != 0:
            raise RuntimeError("bench_empty failed")
        b.record()
        torch.cuda.synchronize()
        if r >= 3:
            times.append(a.elapsed_time(b) * 1e3)
    times.sort()
    return round(times[len(times) // 2], 2)


STREAM_MODES = {"read": 0, "write": 1, "copy": 2, "fanout": 3, "fanin": 4}


def bench_stream(mode, dst, src, nbytes, k=1, grid=1024, sink=None, stream=None):
    import torch
    s = (stream or torch.cuda.current_stream()).cuda_stream
    rc = bench_kernels().bench_stream(STREAM_MODES[mode], ctypes.c_void_p(dst.data_ptr() if dst is not None else 0),
                                      ctypes.c_void_p(src.data_ptr() if src is not None else 0), ctypes.c_size_t(nbytes),
                                      int(k), int(grid), ctypes.c_void_p(sink.data_ptr() if sink is not None else 0),
                                      ctypes.c_void_p(int(s)))
    if rc != 0:
        raise RuntimeError(f"bench_stream({mode}) failed with {rc}")


def stream_ceilings(part=256 << 20, reps=8, grids=(256, 512, 1024, 2048, 4096)):
    """GB/s of plain streaming kernels with the executor's access pattern, best grid each: read only, write only,
    copy, one read fanned out to 7 writes, 8 reads summed into one write.  `part` bytes per region, 8 regions."""
    import torch
    a = torch.empty(8 * part, dtype=torch.uint8, device="cuda:0").random_(0, 255)
    b = torch.empty(8 * part, dtype=torch.uint8, device="cuda:0")
    sink = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    cases = {"read": ("read", 8 * part, 1, 8 * part), "write": ("write", 8 * part, 1, 8 * part),
             "copy": ("copy", 8 * part, 1, 16 * part), "fanout_1r_7w": ("fanout", part, 7, 8 * part),
             "fanin_8r_1w": ("fanin", part, 8, 9 * part)}
    out = {}
    for name, (mode, nbytes, k, traffic) in cases.items():
        best = None
        for grid in grids:
            times = []
            for r in range(reps + 1):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                bench_stream(mode, b, a, nbytes, k, grid, sink)
                e1.record()
                torch.cuda.synchronize()
                if r:
                    times.append(e0.elapsed_time(e1))
            med = sorted(times)[len(times) // 2]
            if best is None or med < best[0]:
                best = (med, grid)
        out[name] = {"GBs": round(traffic / (best[0] * 1e-3) / 1e9, 1), "grid": best[1], "ms": round(best[0], 4),
                     "bytes": traffic}
    return out


# ---- traffic behind the L2, from the committed rocprofv3 summaries under profiles/

def measured_traffic(workload, st):
    """(bytes per launch, source) from the `traffic:` line of a profile summary whose workload and launch shape match
    this run's, else (None, None).  The numbers were measured by builder-run `rocprofv3 --pmc` passes (commands in
    the file), not in this process."""
    want = {"workload": workload, "lowering": LOWERING_NAMES.get(st["lowering"], "?"), "grid": str(st["grid_workgroups"])}
    if st["lowering"] == 1:
        want.update({"block_threads": str(st["block_threads"]), "vectors_per_thread": str(st["vectors_per_thread"])})
    else:
        want.update({"slice_vectors": str(st["slice_vectors"]), "staged_threads": str(st["staged_threads"])})
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*.md"))):
        with open(path) as f:
            for line in f:
                if not line.startswith("traffic:"):
                    continue
                kv = dict(re.findall(r"(\w+)=(\S+)", line))
                if all(kv.get(k) == v for k, v in want.items()) and "fetch_bytes" in kv and "write_bytes" in kv:
                    return float(kv["fetch_bytes"]) + float(kv["write_bytes"]), f"profiles/{os.path.basename(path)} (builder-run rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE)"
    return None, None


def roofline(workload, st, mean_ms):
    """The roofline object of the JSON line.  `achieved` follows the metric: ALGORITHMIC bytes (every chunk move of
    the schedule: a copy group reads 1 and writes k chunks, a reduce group reads k + 1 and writes 1) over the
    kernel's mean duration.  A lane re-reads in step s+1 what it wrote in step s, and those re-reads are served by
    the L2, so the bytes that actually cross to HBM are fewer: `traffic` (counters), bounded below by
    `compulsory_bytes` (every cell read before it is written is fetched once, every cell written is written once)."""
    t = mean_ms * 1e-3
    gbs = st["bytes_min"] / t / 1e9
    compulsory = (st["num_cells_loaded"] + st["num_cells_stored"]) * st["chunk_bytes"]
    traffic, source = measured_traffic(workload, st)
    r = {"bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(gbs / HBM_PEAK_GBS, 4),
         "traffic": traffic, "traffic_frac": None if traffic is None else round(traffic / t / 1e9 / HBM_PEAK_GBS, 4),
         "traffic_source": source,
         "compulsory_bytes": compulsory, "compulsory_frac": round(compulsory / t / 1e9 / HBM_PEAK_GBS, 4),
         "kernel": ("sccl_staged_kernel" if st["lowering"] == 2 else "sccl_exec_kernel") + " (one launch = the whole schedule)",
         "kernel_ms": round(mean_ms, 4), "algorithmic_bytes_per_launch": st["bytes_min"],
         "note": "frac = algorithmic bytes / time / peak, the metric's definition.  It is not a fraction of HBM traffic: "
                 "re-reads of what a lane wrote one step earlier hit the L2, so frac can exceed traffic_frac (bytes counted "
                 "behind the L2) and even 1.  compulsory_frac uses only the bytes any execution must move."}
    return r


# ---- running a workload

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


_flush = None


def flush_caches():
    """READS 1 GiB of scratch memory: whatever the L2s (8 x 4 MiB) and the memory-side cache (256 MiB) held of the
    working set is evicted (and, where dirty, written back) before the timed launch starts, and what replaces it is
    clean -- a flush that wrote would leave its own dirty lines to be written back during the timed launch.
    Enqueued on the current stream, outside every timed window."""
    global _flush
    import torch
    if _flush is None:
        _flush = (torch.zeros(1 << 30, dtype=torch.uint8, device="cuda:0"), torch.zeros(1, dtype=torch.int32, device="cuda:0"))
    bench_stream("read", None, _flush[0], 1 << 30, grid=1024, sink=_flush[1])


def time_workload(wl, steps, warmup, options=None, keep=False, mode="sccl_execute", cold=False, cold_steps=0, memory=None):
    """Returns dict with per-step kernel times (ms) measured by events on the launch stream.  cold: the caches are
    flushed between restoring the inputs and the timed launch (else the restore's writes may still sit in them).
    cold_steps: that many further launches with flushed caches ON THE SAME BUFFERS ("ms_cold"): a new allocation
    gets other physical pages, which alone moves the largest workloads by several percent either way.
    memory: (pristine, work) of an earlier run of the same sizes, to be used again for the same reason."""
    import torch
    from paper_2008_08708_amd import schedule_file, sccl
    dev = torch.device("cuda:0")
    sf = schedule_file.load(wl.schedule)
    if wl.options:                                   # the workload's own launch shape, unless the caller names one
        options = {**wl.options, **(options or {})}
    pristine, epc = make_inputs(wl, sf, dev)
    if memory is None:
        work = [torch.empty_like(b) for b in pristine]
    else:
        for old, new in zip(memory[0], pristine):
            old.copy_(new)
        pristine, work = memory
    plan = sccl.sccl_plan_create(*sf.descriptions(wl.dtype, epc), options=options)
    stats = sccl.sccl_plan_stats(plan)
    stream = torch.cuda.current_stream()
    execute = getattr(sccl, mode)

    def restore():
        for w, p in zip(work, pristine):
            w.copy_(p)
        if cold:
            flush_caches()

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
    if cold_steps:
        cevs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(cold_steps)]
        for a, b in cevs:
            restore()
            if not cold:
                flush_caches()
            a.record(stream)
            execute(plan, work, stream)
            b.record(stream)
        torch.cuda.synchronize()
        out["ms_cold"] = [a.elapsed_time(b) for a, b in cevs]
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


def cpu_baseline(run, wl):
    """The oracle, as it stands, on the host cores: the full workload, same plan, same input bits.
    Also compares the GPU's result with it, bit for bit, on the full buffers."""
    import numpy as np
    import torch
    from oracle import executor, schedule as osched
    from paper_2008_08708_amd import sccl
    sf, epc = run["sf"], run["epc"]
    sched = osched.Schedule(sf.rounds, sf.sends)
    nproc = os.cpu_count() or 1
    threads = max(1, min(nproc, executor.max_threads()))     # every core OpenMP may use (OMP_NUM_THREADS caps it)
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
    return {"value": run["stats"]["bytes_min"] / med / 1e9, "unit": "GB/s", "cores": threads, "nproc": nproc, "kind": "oracle",
            "value_one_core": run["stats"]["bytes_min"] / one / 1e9,
            "sample": f"the full workload ({run['stats']['bytes_min'] / 2**30:.2f} GiB algorithmic), median of 3 runs, "
                      f"OpenMP over the element range on {threads} threads (the host reports {nproc} processors)"}, same


def sweep(wl, steps, warmup):
    """Every launch shape of the through-memory kernel (workgroup size x vectors per lane x workgroups per CU) and,
    where the cells fit, of the staged kernel (slice x workgroup size); one JSON line each, the best last."""
    from paper_2008_08708_amd import sccl
    shapes = [{"lowering": 1, "block_threads": bt, "vectors_per_thread": vt, "max_workgroups": 256 * k}
              for bt in (64, 128, 256) for vt in (1, 2, 4, 8) for k in (1, 2, 4)]
    shapes += [{"lowering": 2, "slice_vectors": sv, "staged_threads": th}
               for sv in (1, 2, 4, 8, 16, 32, 64, 128) for th in (64, 256, 512, 1024)]
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


def crossover(steps, warmup):
    """Both lowerings of sccl_execute on twelve schedules at total sizes from 64 KiB to 256 MiB (all ranks together),
    and which one SCCL_LOWER_AUTO picks: the evidence behind the automatic choice.  One JSON line per (schedule,
    size); `auto_is_best` allows 3 % of noise."""
    import dataclasses
    from paper_2008_08708_amd import schedule_file, sccl, workloads
    names = ["cfg1", "cfg2", "cfg3", "cfg4b", "alltoall", "broadcast", "reduce", "gather"]
    wls = [workloads.WORKLOADS[k] for k in names]
    wls += [workloads.sweep_workload(c, 1024, a) for c in ("allgather", "allreduce") for a in ("bandwidth", "latency")]
    wrong = 0
    for wl in wls:
        sf = schedule_file.load(wl.schedule)
        unit = sf.num_nodes * sf.positions_per_rank * 16                       # one 16-byte vector per chunk position
        for total in [1 << e for e in range(16, 29, 2)]:
            per_rank = max(1, total // unit) * sf.positions_per_rank * 16
            w = dataclasses.replace(wl, bytes_per_rank=per_rank, options=None)      # the plan's own launch shape at every size
            res = {}
            for key, low in (("auto", 0), ("memory", 1), ("staged", 2)):
                try:
                    r = time_workload(w, steps, warmup, {"lowering": low} if low else None)
                except sccl.ScclError:
                    res[key] = None
                    continue
                m = sorted(r["ms"])
                res[key] = round(m[len(m) // 2] * 1e3, 2)
                if key == "auto":
                    st = r["stats"]
            best = min(v for k, v in res.items() if k != "auto" and v is not None)
            ok = res["auto"] <= 1.03 * best + 0.3
            wrong += not ok
            print(json.dumps({"schedule": wl.schedule, "total_bytes": per_rank * sf.num_nodes, "auto": LOWERING_NAMES[st["lowering"]],
                              "us_auto": res["auto"], "us_memory": res["memory"], "us_staged": res["staged"],
                              "groups_per_chunk": st["max_chunk_groups"], "levels": st["num_levels"],
                              "staged_levels": st["staged_levels"], "staged_items": st["num_slices"], "auto_is_best": ok}), flush=True)
    print(json.dumps({"choices_that_lose_more_than_3_percent": wrong}), flush=True)


def report(path, torch, workloads, sccl):
    """Times every configuration under every lowering, warm and cold, beside the oracle; the torus pair the
    cost model chooses between; and the streaming ceilings.  Markdown to `path`."""
    from paper_2008_08708_amd.sccl import SCCL_LOWER_MEMORY, SCCL_LOWER_STAGED, ScclError
    rows = []
    names = [(k, workloads.WORKLOADS[k]) for k in ("cfg1", "cfg2", "cfg3", "cfg4", "cfg4b", "alltoall", "broadcast", "reduce",
                                                   "gather", "scatter", "reducescatter")]
    for coll in ("allgather", "allreduce"):
        for size in workloads.sweep_sizes():
            names.append((f"cfg5 {coll} {size}", workloads.sweep_workload(coll, size)))

    def median_us(w, steps, mode, opts=None, cold_steps=0):
        r = time_workload(w, steps, 3, options=opts, mode=mode, cold_steps=cold_steps)
        m = sorted(r["ms"])
        out = (m[len(m) // 2] * 1e3, m[0] * 1e3, r["stats"])
        if cold_steps:
            mc = sorted(r["ms_cold"])
            out += (mc[len(mc) // 2] * 1e3,)
        del r
        torch.cuda.empty_cache()
        return out

    fmt = lambda x: "-" if x is None else format(x, ".1f")
    for label, w in names:
        steps = 5 if w.bytes_per_rank >= (1 << 30) else 20
        # the default (lowering chosen by the plan), then cold caches on the same buffers
        med, mn, s, cold_med = median_us(w, steps, "sccl_execute", cold_steps=steps)
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
        rf = roofline(w.name, s, med * 1e-3)
        rows.append((label, s["num_nodes"], w.bytes_per_rank, s["chunk_bytes"], s["num_steps"], s["bytes_min"],
                     med, mn, s["bytes_min"] / (med * 1e-6) / 1e9, "staged" if s["lowering"] == SCCL_LOWER_STAGED else "memory",
                     f'{s["num_levels"]} ({s["staged_levels"]})', s["grid_workgroups"], mem_med, stg_med, step_med, cpy_med, graph_us, oracle, cold_med, rf))
        print(f"[report] {label}: default ({rows[-1][9]}) {med:.1f} us warm, {cold_med:.1f} us cold ({rows[-1][8]:.1f} GB/s), "
              f"through memory {fmt(mem_med)} us, staged {fmt(stg_med)} us, per-step kernels {fmt(step_med)} us, "
              f"per-send copies {fmt(cpy_med)} us, in a graph of 20 {fmt(graph_us)} us each", file=sys.stderr, flush=True)
    os.makedirs(os.path.dirname(os.path.abspath(path)), exist_ok=True)
    with open(path, "w") as f:
        f.write("`python bench.py --report FILE` on one MI355X (3 warm-up + 20 timed launches per figure, 5 at 16 GiB): every workload under the default lowering, warm and "
                "with cold caches, each lowering forced, the paper's other two lowerings, and the oracle on the host.  Medians of "
                "the time between HIP events around one execute call, microseconds.\n\n")
        f.write("| workload | P | bytes/rank | chunk bytes | S | bytes_min | sccl_execute: median us | min us | cold caches: median us "
                "| effective GB/s | algorithmic % of 8 TB/s | compulsory % of 8 TB/s "
                "| lowering | dependency levels (left when staged) | grid | through memory: us | staged: us | one kernel per step: us | one copy per send: us "
                "| each of 20 in one HIP graph: us | oracle on the host cores: GB/s (cores) | oracle on one core: GB/s "
                "| full buffers bitwise equal to the oracle's |\n")
        f.write("|" + "---|" * 23 + "\n")
        for r in rows:
            f.write(f"| {r[0]} | {r[1]} | {r[2]} | {r[3]} | {r[4]} | {r[5]} | {r[6]:.1f} | {r[7]:.1f} | {r[18]:.1f} | {r[8]:.1f} | "
                    f"{100 * r[19]['frac']:.1f} | {100 * r[19]['compulsory_frac']:.1f} | {r[9]} | {r[10]} | {r[11]} | {fmt(r[12])} | {fmt(r[13])} | "
                    f"{fmt(r[14])} | {fmt(r[15])} | {fmt(r[16])} | "
                    + ("- | - | (every byte: tests/test_gpu_fullsize.py) |\n" if r[17] is None else
                       f"{r[17][0]:.1f} ({r[17][2]}) | {r[17][1]:.1f} | {'yes' if r[17][3] else 'NO'} |\n"))
    # ---- the paper's size-dependent choice between two algorithms (section 5.5) on this hardware: the
    # latency-optimal and the bandwidth-optimal torus algorithm at every size, and what two fits of the cost model
    # would have chosen: the paper's t = S alpha + (R/C) L beta, and the same with a launch intercept t0.
    with open(path, "a") as f:
        f.write("\n| collective | bytes/rank | latency-optimal: us | bandwidth-optimal: us | measured best (tie: within 3 %) "
                "| paper's model chooses | model with intercept, fitted to relative errors, chooses |\n|---|---|---|---|---|---|---|\n")
        score = {"paper": 0, "intercept": 0, "rows": 0}
        for coll in ("allgather", "allreduce"):
            meas = []
            for size in workloads.sweep_sizes():
                pair = []
                memory = None                                      # both algorithms run in the same device memory
                for alg in ("latency", "bandwidth"):
                    w = workloads.sweep_workload(coll, size, alg)
                    steps = 5 if size >= (1 << 30) else 20
                    r = time_workload(w, steps, 3, keep=True, memory=memory)
                    memory = (r["pristine"], r["work"])
                    sccl.sccl_plan_destroy(r["plan"])
                    m, st_ = sorted(r["ms"]), r["stats"]
                    # the model's two coordinates: a = S, b = (R / C) * L = R * chunk bytes
                    pair.append((m[len(m) // 2] * 1e-3, float(st_["num_steps"]), float(st_["num_rounds"]) * st_["chunk_bytes"]))
                    del r
                del memory
                torch.cuda.empty_cache()
                meas.append((size, pair))
            a = [p[1] for _, pair in meas for p in pair]
            b = [p[2] for _, pair in meas for p in pair]
            t = [p[0] for _, pair in meas for p in pair]
            alpha, beta = sccl.sccl_cost_fit(a, b, t)
            t0, alpha3, beta3 = sccl.sccl_cost_fit_intercept(a, b, t, weights=[1.0 / x for x in t])    # relative errors
            for size, pair in meas:
                model = [p[1] * alpha + p[2] * beta for p in pair]
                model3 = [t0 + p[1] * alpha3 + p[2] * beta3 for p in pair]
                best = "latency" if pair[0][0] <= pair[1][0] else "bandwidth"
                if abs(pair[0][0] - pair[1][0]) <= 0.03 * min(pair[0][0], pair[1][0]):
                    best = "tie"                                   # within 3 %: the same lowering measured twice differs by as much
                c2 = "latency" if model[0] <= model[1] else "bandwidth"
                c3 = "latency" if model3[0] <= model3[1] else "bandwidth"
                score["rows"] += 1
                score["paper"] += best in ("tie", c2)
                score["intercept"] += best in ("tie", c3)
                f.write(f"| {coll} | {size} | {pair[0][0] * 1e6:.1f} | {pair[1][0] * 1e6:.1f} | {best} | {c2} | {c3} |\n")
            f.write(f"\n{coll}: paper's model alpha = {alpha * 1e6:.3f} us per step, 1 / beta = "
                    f"{1e-9 / beta if beta > 0 else float('inf'):.0f} GB/s; with intercept t0 = {t0 * 1e6:.2f} us, alpha = "
                    f"{alpha3 * 1e6:.3f} us per step, 1 / beta = {1e-9 / beta3 if beta3 > 0 else float('inf'):.0f} GB/s\n")
            print(f"[report] {coll}: alpha {alpha * 1e6:.3f} us, beta {beta * 1e12:.4f} ps/B; with intercept t0 {t0 * 1e6:.2f} us, "
                  f"alpha {alpha3 * 1e6:.3f} us, beta {beta3 * 1e12:.4f} ps/B", file=sys.stderr, flush=True)
        f.write(f"\nChoices that are the measured best or a tie, out of {score['rows']}: the paper's model {score['paper']}, the model "
                f"with a launch intercept {score['intercept']}.\n")
        ceil = stream_ceilings()
        f.write("\n| plain streaming kernel (256 MiB regions) | GB/s | % of 8 TB/s | best grid |\n|---|---|---|---|\n")
        for k, v in ceil.items():
            f.write(f"| {k} | {v['GBs']:.0f} | {100 * v['GBs'] / HBM_PEAK_GBS:.1f} | {v['grid']} |\n")
        f.write("\nContext, not a target: the paper gives no absolute time or bandwidth for executing a schedule in its "
                "text, only speedups measured across eight GPUs over their links (section 5.5): Allgather up to 2.2x "
                "(small) and 1.14x (large) over NCCL 2.7.8, Allreduce up to 1.8x (small, the 8-chunk algorithm) and 1.06x "
                "(large, the 48-chunk algorithm), Alltoall more than 6.8x (large) over point-to-point copies, on a DGX-1 "
                "(8 x V100, six 25 GB/s NVLink ports per GPU); Allgather faster than RCCL only at large sizes on a Gigabyte "
                "Z52 (8 x MI50, xGMI about 33 GB/s, PCIe 4 about 27 GB/s).  Nothing here reproduces an inter-GPU link: the "
                "figures above are one MI355X moving P virtual ranks' buffers inside its own HBM "
                f"(peak {HBM_PEAK_GBS / 1000:.0f} TB/s).\n")


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
    ap.add_argument("--slice-vectors", type=int, default=0)
    ap.add_argument("--staged-threads", type=int, default=0)
    ap.add_argument("--cold", action="store_true",
                    help="flush the caches (a 1 GiB scratch read) between restoring the inputs and every timed launch")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-ceilings", action="store_true", help="skip the plain streaming kernels")
    ap.add_argument("--ceilings", action="store_true", help="only measure the plain streaming kernels; one JSON line")
    ap.add_argument("--report", default="", metavar="FILE", help="also time the other configurations; markdown table to FILE")
    ap.add_argument("--crossover", action="store_true",
                    help="instead of the benchmark line: both lowerings on twelve schedules over a range of sizes, one JSON line each")
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
    if args.ceilings:
        print(json.dumps({"streaming_ceilings": stream_ceilings(), "peak_GBs": HBM_PEAK_GBS,
                          "empty_kernel_us_between_events": {str(g): launch_floor_us(g) for g in (64, 256, 4096, 16384, 65536)}}), flush=True)
        return
    options = {k: v for k, v in (("block_threads", args.block_threads), ("vectors_per_thread", args.vectors_per_thread),
                                 ("max_workgroups", args.max_workgroups), ("lowering", args.lowering),
                                 ("slice_vectors", args.slice_vectors), ("staged_threads", args.staged_threads)) if v}
    if args.workload.startswith("cfg5:"):             # cfg5:<allgather|allreduce>:<bytes per rank>[:latency]
        parts = args.workload.split(":")
        wl = workloads.sweep_workload(parts[1], int(parts[2]), parts[3] if len(parts) > 3 else "bandwidth")
    else:
        wl = workloads.WORKLOADS[args.workload]
    if args.crossover:
        crossover(args.steps, args.warmup)
        return
    if args.sweep:
        sweep(wl, args.steps, args.warmup)
        return
    run = time_workload(wl, args.steps, args.warmup, options or None, keep=True, cold=args.cold)
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
                   "lowering": LOWERING_NAMES.get(st["lowering"]), "grid": st["grid_workgroups"],
                   "block_threads": st["block_threads"], "vectors_per_thread": st["vectors_per_thread"],
                   "caches": "flushed before every timed launch" if args.cold else "as the restore of the inputs left them"},
        "pct_of_hbm_peak": round(100.0 * gbs / HBM_PEAK_GBS, 2),
        "ms_min": round(min(ms), 4), "ms_median": round(sorted(ms)[len(ms) // 2], 4),
        "wall_ms_per_step_incl_restore": round(run["wall_s"] * 1e3 / args.steps, 4),
        "roofline": roofline(wl.name, st, mean_ms),
    }
    if not args.cold and not args.no_ceilings:
        # the same kernel with cold caches (untimed region: restore + 1 GiB scratch read), a few steps
        for w, p in zip(run["work"], run["pristine"]):
            w.copy_(p)
        cold = []
        for _ in range(min(5, args.steps)):
            for w, p in zip(run["work"], run["pristine"]):
                w.copy_(p)
            flush_caches()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            sccl.sccl_execute(run["plan"], run["work"])
            b.record()
            torch.cuda.synchronize()
            cold.append(a.elapsed_time(b))
        line["ms_per_step_cold_caches"] = round(sum(cold) / len(cold), 4)
    if not args.no_ceilings:
        try:
            c = stream_ceilings(reps=4, grids=(1024, 2048))
            line["streaming_ceilings_gbs"] = {k: v["GBs"] for k, v in c.items()}
            line["empty_kernel_us_between_events"] = launch_floor_us()
        except Exception as e:                    # measurement aid only
            line["streaming_ceilings_gbs"] = None
            print(f"streaming ceilings failed: {e}", file=sys.stderr)
    if not args.no_cpu_baseline:
        base, same = cpu_baseline(run, wl)
        line["cpu_baseline"] = base
        line["parity_full_buffers_bitwise"] = bool(same)
    sccl.sccl_plan_destroy(run["plan"])
    del run
    torch.cuda.empty_cache()
    if args.report:
        report(args.report, torch, workloads, sccl)
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
