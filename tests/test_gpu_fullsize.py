"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times (the plan's own choice, or the workload's
stored launch shape where it has one): every
configuration of the measurement -- configurations 1, 2, 3, 4 (both readings), all eleven sizes of configuration 5
for both collectives, the latency-optimal torus pair, and Alltoall, Broadcast, Reduce, Gather, Scatter.

Every byte of every rank buffer is compared, at 0 ulp, in two ways:

  * with the CPU oracle, element range by element range.  Elements are independent, so running the schedule on a
    range of every chunk (the same input bits, read back from the device before the run) must give the bits the
    GPU left in that range.  The ranges tile the whole buffers (32 MiB over all ranks per range, so host memory
    stays small whatever the working set); they are visited first, ragged last, then in a seeded random order.
    On the 16-core test box the oracle gets through every range of every case (the 16 GiB torus Allreduce: 63 GB
    of algorithmic bytes) in about a second, most of a case's time being the transfers; ORACLE_SECONDS is only a
    guard for a slower host (the share covered is printed, and SCCL_FULL_ORACLE=1 lifts it).
  * with a second executor made of plain PyTorch operations on the device (tests/device_reference.py), on the
    whole buffers, always.

On top: the closed form of every non-combining collective on the whole buffers (wherever post wants chunk c it is
the chunk of its holder in pre), all ranks bitwise equal after Allreduce, and the lowering the plan chose on each
side of the measured crossover of configuration 5.  Tolerance: 0 ulp (see test_gpu_parity.py).
"""
import os
import time

import numpy as np
import pytest

import device_reference
from oracle import executor as ex
from oracle.schedule import Schedule
from paper_2008_08708_amd import schedule_file, sccl, workloads
from bench import make_inputs

pytestmark = pytest.mark.gpu

FULL = os.environ.get("SCCL_FULL_ORACLE", "") not in ("", "0")
ORACLE_SECONDS = 10.0                                            # oracle time per case before the remaining ranges are skipped
RANGE_BYTES = 32 << 20                                           # one range over all ranks and chunk positions: cache sized

CASES = [(k, workloads.WORKLOADS[k]) for k in ("cfg1", "cfg2", "cfg3", "cfg4", "cfg4b", "alltoall", "broadcast", "reduce",
                                               "gather", "scatter", "reducescatter")]
for coll in ("allgather", "allreduce"):
    for size in workloads.sweep_sizes():                         # all eleven sizes of configuration 5
        CASES.append((f"cfg5-{coll}-{size}", workloads.sweep_workload(coll, size)))
    for size in (1 << 10, 1 << 20, 1 << 28):                     # the latency-optimal algorithm the selection is measured with
        CASES.append((f"cfg5-{coll}-latency-{size}", workloads.sweep_workload(coll, size, "latency")))


def element_ranges(epc, ranks, positions, elem_bytes, seed):
    """(start, count) ranges that tile a chunk's elements, in visiting order: first, last (ragged), the rest shuffled."""
    count = max(1, RANGE_BYTES // (ranks * positions * elem_bytes))
    starts = list(range(0, epc, count))
    order = [starts[0]] + ([starts[-1]] if len(starts) > 1 else [])
    rest = starts[1:-1]
    np.random.default_rng(seed).shuffle(rest)
    return [(st, min(count, epc - st)) for st in order + rest]


@pytest.mark.parametrize("label,wl", CASES, ids=[c[0] for c in CASES])
def test_full_size_every_byte(label, wl):
    import torch
    print(f"[case] {label}: {wl.schedule} {wl.bytes_per_rank} bytes/rank {wl.dtype}", flush=True)
    sf = schedule_file.load(wl.schedule)
    P, G, K = sf.num_nodes, sf.num_chunks, sf.positions_per_rank
    pristine, epc = make_inputs(wl, sf, torch.device("cuda:0"))
    work = [p.clone() for p in pristine]
    plan = sccl.sccl_plan_create(*sf.descriptions(wl.dtype, epc), options=wl.options)
    st = sccl.sccl_plan_stats(plan)
    if label.startswith("cfg5-") and "latency" not in label:    # the measured crossover of the automatic lowering
        staged_up_to = (4 << 20) if "allgather" in label else (1 << 20)
        want_lowering = sccl.SCCL_LOWER_STAGED if wl.bytes_per_rank <= staged_up_to else sccl.SCCL_LOWER_MEMORY
        assert st["lowering"] == want_lowering, (wl.bytes_per_rank, st["lowering"])
    sccl.sccl_execute(plan, work)
    torch.cuda.synchronize()
    sccl.sccl_plan_destroy(plan)
    u = np.uint32 if wl.elem_bytes == 4 else np.uint16
    tu = torch.int32 if wl.elem_bytes == 4 else torch.int16

    # ---- the oracle, range by range
    ranges = element_ranges(epc, P, K, wl.elem_bytes, seed=wl.seed)
    sched = Schedule(sf.rounds, sf.sends)
    layout = {} if sf.slot is None else {"slot": sf.slot, "slots_per_rank": sf.slots_per_rank}
    before = torch.stack([p.view(K, epc) for p in pristine]) if P * wl.bytes_per_rank <= (64 << 20) else None
    covered, spent, done = 0, 0.0, 0
    for start, count in ranges:
        if not FULL and done >= 2 and spent > ORACLE_SECONDS:
            break
        if before is not None:
            host_all = before[:, :, start:start + count].contiguous().cpu().numpy()
        else:
            host_all = torch.stack([p.view(K, epc)[:, start:start + count] for p in pristine]).cpu().numpy()
        host = [host_all[n].reshape(-1) for n in range(P)]
        t0 = time.perf_counter()
        ex.execute(wl.dtype, G, count, sched, host, threads=16, **layout)
        spent += time.perf_counter() - t0
        got_all = torch.stack([w.view(K, epc)[:, start:start + count] for w in work]).cpu().numpy()
        for n in range(P):
            got = got_all[n].reshape(-1)
            bad = np.nonzero(got.view(u) != host[n].view(u))[0]
            assert bad.size == 0, (f"rank {n}: {bad.size} elements of range [{start}, {start + count}) differ from the oracle, "
                                   f"first at position {bad[0] // count} element {start + bad[0] % count}")
        covered += count
        done += 1
    print(f"[case]   oracle: {done} of {len(ranges)} ranges, {covered} of {epc} elements per chunk "
          f"({100.0 * covered / max(1, epc):.1f} % of every buffer) in {spent:.1f} s of oracle time", flush=True)

    # ---- the device reference, every byte
    ref = [p.clone() for p in pristine]
    device_reference.execute(sf, wl.dtype, epc, ref)
    torch.cuda.synchronize()
    for n in range(P):
        same = torch.equal(work[n].view(tu), ref[n].view(tu))
        if not same:
            bad = torch.nonzero(work[n].view(tu) != ref[n].view(tu))
            raise AssertionError(f"rank {n}: {bad.shape[0]} elements differ from the device reference, first at {int(bad[0])}")
    del ref

    # ---- properties of the whole buffers
    def position(c, n):
        return c if sf.slot is None else int(sf.slot[c, n])

    if not sf.combining:                                   # closed form of every non-combining collective (Table 2)
        for c in range(G):
            holder = int(np.nonzero(sf.pre[c])[0][0])
            src = pristine[holder].view(K, epc)[position(c, holder)].view(tu)
            for n in range(P):
                if sf.post[c, n]:
                    assert torch.equal(work[n].view(K, epc)[position(c, n)].view(tu), src), f"chunk {c} at rank {n}"
    elif sf.collective == "allreduce":
        for n in range(1, P):
            assert torch.equal(work[n].view(tu), work[0].view(tu)), f"rank {n} differs from rank 0"
        assert not torch.isnan(work[0]).any()
    else:                                                  # Reduce, Reducescatter: no NaN where post puts the sum
        for c in range(G):
            for n in range(P):
                if sf.post[c, n]:
                    assert not torch.isnan(work[n].view(K, epc)[position(c, n)]).any()


def test_reduce_at_the_root_in_closed_form():
    """Exact inputs (small integers: every order of addition gives the same binary32 bits): after Reduce the root
    holds the plain sum over the ranks, on the whole buffer."""
    import torch
    from paper_2008_08708_amd import inputs
    wl = workloads.WORKLOADS["reduce"]
    sf = schedule_file.load(wl.schedule)
    P, G = sf.num_nodes, sf.num_chunks
    n_elems = wl.bytes_per_rank // 4
    epc = n_elems // G
    bufs = [inputs.torch_rank_buffer("smallint", "f32", 8, n, n_elems, torch.device("cuda:0")) for n in range(P)]
    total = torch.zeros(n_elems, dtype=torch.float32, device="cuda:0")
    for b in bufs:
        total += b
    plan = sccl.sccl_plan_create(*sf.descriptions("f32", epc))
    print(f"[case] reduce closed form, {n_elems} elements per rank", flush=True)
    sccl.sccl_execute(plan, bufs)
    torch.cuda.synchronize()
    sccl.sccl_plan_destroy(plan)
    for c in range(G):
        for n in range(P):
            if sf.post[c, n]:
                assert torch.equal(bufs[n].view(G, epc)[c], total.view(G, epc)[c]), f"chunk {c} at root {n}"


@pytest.mark.parametrize("mode,lowering", [("sccl_execute", sccl.SCCL_LOWER_MEMORY), ("sccl_execute", sccl.SCCL_LOWER_STAGED),
                                           ("sccl_execute_stepwise", 0)])
def test_chunks_larger_than_four_gibibytes(mode, lowering):
    """Byte offsets inside one chunk beyond 32 bits: Allreduce between two ranks, two chunks of 4 GiB + 4 MiB + 592 B
    each (a ragged last tile), 16 GiB in all.  Two operands: the sum has the same bits in either order, so the
    whole result is checked on the device against in_0 + in_1; the oracle checks ranges at the start of a chunk,
    across the 4 GiB offset and at the ragged end."""
    import torch
    from helpers import to_binding
    from oracle import collective as col, generate as gen, topology as tp
    from paper_2008_08708_amd import inputs
    topo = tp.point_to_point(2, {(0, 1): 1, (1, 0): 1}, "pair")
    ag = col.allgather(2, 1)
    sched, coll = gen.compose_allreduce(gen.greedy_bfs(topo, ag), ag)
    epc = (1 << 30) + (1 << 20) + 4 * 37
    dev = torch.device("cuda:0")
    pristine = [inputs.torch_rank_buffer("uniform", "f32", 77, n, 2 * epc, dev) for n in range(2)]
    work = [p.clone() for p in pristine]
    plan = sccl.sccl_plan_create(*to_binding(topo, coll, sched, "f32", epc), options={"lowering": lowering} if lowering else None)
    st = sccl.sccl_plan_stats(plan)
    assert st["chunk_bytes"] > (1 << 32) and st["vector_bytes"] == 16
    print(f"[case] chunks of {st['chunk_bytes']} bytes, {mode}, lowering={lowering}", flush=True)
    getattr(sccl, mode)(plan, work)
    torch.cuda.synchronize()
    sccl.sccl_plan_destroy(plan)
    want = pristine[0] + pristine[1]
    for n in range(2):
        assert torch.equal(work[n].view(torch.int32), want.view(torch.int32)), f"rank {n}"
    del want
    osched = Schedule(sched.rounds, sched.sends)
    for start, count in ((0, 4096), ((1 << 30) - 2048, 4096), (epc - 4099, 4099)):
        host = [torch.stack([p.view(2, epc)[c, start:start + count] for c in range(2)]).reshape(-1).cpu().numpy() for p in pristine]
        ex.execute("f32", 2, count, osched, host)
        for n in range(2):
            got = torch.stack([work[n].view(2, epc)[c, start:start + count] for c in range(2)]).reshape(-1).cpu().numpy()
            assert (got.view(np.uint32) == host[n].view(np.uint32)).all(), (n, start)
