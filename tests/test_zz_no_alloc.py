"""sccl_execute_static, the entry point that allocates nothing, against sccl_execute.

Both run the same kernels; the static one reads the step table from the library's static device array,
which every call on the GPU shares and which keeps the last call's contents.  So every case here makes
TWO calls in a row, the second with a smaller input (a shorter table, fewer elements, or both), and
compares each call's buffers bit for bit with what sccl_execute leaves on the same inputs (and with the
oracle).  Plans are SCCL_PLAN_HOST_ONLY where noted: such a plan never touched the device, so nothing in
the static path can be using memory a plan allocated.
"""
import numpy as np
import pytest

from oracle import executor as ex
from oracle.schedule import Schedule
from paper_2008_08708_amd import inputs, schedule_file, sccl

pytestmark = pytest.mark.gpu

M, S = sccl.SCCL_LOWER_MEMORY, sccl.SCCL_LOWER_STAGED

# (label, [(schedule, dtype, dist, elems per chunk, lowering, host-only plan), (the same for the second, smaller call)])
CASES = [
    ("memory-f32-then-fewer-elements", [("cfg3_allreduce_hcm8", "f32", "uniform", 70001, M, True),
                                        ("cfg3_allreduce_hcm8", "f32", "uniform", 1003, M, True)]),
    ("staged-f32-then-fewer-elements", [("cfg5_allreduce_torus4x4", "f32", "uniform", 260, S, True),
                                        ("cfg5_allreduce_torus4x4", "f32", "uniform", 40, S, True)]),
    ("long-table-then-short-table", [("cfg5_allreduce_torus4x4", "f32", "uniform", 4100, M, True),
                                     ("cfg1_allgather_ring4", "f32", "uniform", 1024, M, True)]),
    ("staged-then-memory-f16", [("cfg4_allreduce_ring8", "f16", "normal", 2056, S, False),
                                ("cfg4b_allreduce_ring8_c2", "f16", "normal", 520, M, False)]),
    ("memory-i32-then-staged", [("cfg2_allgather_hcm8", "i32", "u32", 30011, M, False),
                                ("cfg2_allgather_hcm8", "i32", "u32", 64, S, True)]),
    ("alltoall-slots-then-gather", [("alltoall_dgx1", "f32", "uniform", 5000, M, True),
                                    ("gather_dgx1", "f32", "uniform", 300, M, True)]),
]


def bits(a):
    return a.view(np.uint32 if a.dtype.itemsize == 4 else np.uint16)


def one_call(name, dtype, dist, epc, lowering, host_only, seed):
    """Runs the case through both entry points and the oracle; returns nothing, asserts equality of all three."""
    import torch
    sf = schedule_file.load(name)
    P, K = sf.num_nodes, sf.positions_per_rank
    host = [inputs.generate(dist, dtype, seed, n, 0, K * epc) for n in range(P)]
    if not sf.combining:                                   # positions a rank holds nothing in are undefined inputs
        for n in range(P):
            held = {int(c if sf.slot is None else sf.slot[c, n]) for c in range(sf.num_chunks) if sf.pre[c, n]}
            for k in range(K):
                if k not in held:
                    inputs.poison(host[n], k * epc, (k + 1) * epc)
    want = [h.copy() for h in host]
    ex.execute(dtype, sf.num_chunks, epc, Schedule(sf.rounds, sf.sends), want,
               slot=sf.slot, slots_per_rank=sf.slots_per_rank if sf.slot is not None else None)
    desc = sf.descriptions(dtype, epc)
    print(f"[case] {name} {dtype} epc={epc} lowering={lowering} host_only={host_only}", flush=True)
    ref_plan = sccl.sccl_plan_create(*desc, options={"lowering": lowering})
    ref = [torch.from_numpy(h.copy()).cuda() for h in host]
    sccl.sccl_execute(ref_plan, ref)
    opts = {"lowering": lowering}
    if host_only:
        opts["flags"] = sccl.SCCL_PLAN_HOST_ONLY
    plan = sccl.sccl_plan_create(*desc, options=opts)
    st = sccl.sccl_plan_stats(plan)
    assert 0 < st["static_table_bytes"] <= sccl.SCCL_STATIC_SCRATCH_BYTES
    got = [torch.from_numpy(h.copy()).cuda() for h in host]
    sccl.sccl_execute_static(plan, got)
    torch.cuda.synchronize()
    for n in range(P):
        r, g = ref[n].cpu().numpy(), got[n].cpu().numpy()
        bad = np.nonzero(bits(r) != bits(g))[0]
        assert bad.size == 0, f"rank {n}: {bad.size} elements differ from sccl_execute, first at {bad[0]}"
        bad = np.nonzero(bits(want[n]) != bits(g))[0]
        assert bad.size == 0, f"rank {n}: {bad.size} elements differ from the oracle, first at {bad[0]}"
    if host_only:                                          # a host-only plan has no device table of its own
        with pytest.raises(sccl.ScclError) as e:
            sccl.sccl_execute(plan, got)
        assert e.value.name == "SCCL_ERR_DEVICE"
    sccl.sccl_plan_destroy(plan)
    sccl.sccl_plan_destroy(ref_plan)


@pytest.mark.parametrize("label,calls", CASES, ids=[c[0] for c in CASES])
def test_two_calls_in_a_row_equal_sccl_execute(label, calls):
    for i, (name, dtype, dist, epc, lowering, host_only) in enumerate(calls):
        one_call(name, dtype, dist, epc, lowering, host_only, seed=100 + i)


def test_repeated_calls_on_one_stream_and_bad_buffers():
    """Back-to-back calls with alternating plans on one stream (no synchronisation in between): each call
    rewrites the shared table before its kernel, in stream order."""
    import torch
    big = schedule_file.load("cfg3_allreduce_hcm8")
    small = schedule_file.load("cfg1_allgather_ring4")
    pa = sccl.sccl_plan_create(*big.descriptions("i32", 5000), options={"flags": sccl.SCCL_PLAN_HOST_ONLY})
    pb = sccl.sccl_plan_create(*small.descriptions("i32", 700), options={"flags": sccl.SCCL_PLAN_HOST_ONLY})
    ha = [inputs.generate("smallint", "i32", 7, n, 0, 8 * 5000) for n in range(8)]
    hb = [inputs.generate("u32", "i32", 8, n, 0, 4 * 700) for n in range(4)]
    da = [torch.from_numpy(h.copy()).cuda() for h in ha]
    db = [torch.from_numpy(h.copy()).cuda() for h in hb]
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        for _ in range(3):                                 # Allreduce three times in place: the sum times 8, times 8 again
            sccl.sccl_execute_static(pa, da, stream)
            sccl.sccl_execute_static(pb, db, stream)       # Allgather is idempotent
    stream.synchronize()
    total = np.sum(np.stack(ha).astype(np.int64), axis=0)
    want = ((total * 64) & 0xFFFFFFFF).astype(np.uint32)
    for n in range(8):
        assert (da[n].cpu().numpy().view(np.uint32) == want).all()
    for n in range(4):
        g = db[n].cpu().numpy()
        for c in range(4):
            assert (g[c * 700:(c + 1) * 700] == hb[c % 4][c * 700:(c + 1) * 700]).all()
    # the same checks as sccl_execute, and nothing is enqueued when they fail
    with pytest.raises(sccl.ScclError) as e:
        sccl.sccl_execute_static(pb, [db[0], db[1], db[2], db[2]])
    assert e.value.name == "SCCL_ERR_OVERLAP"
    with pytest.raises(sccl.ScclError) as e:
        sccl.sccl_execute_static(pb, [db[0], db[1], db[2], db[3].view(torch.int8)[4:].data_ptr()])
    assert e.value.name == "SCCL_ERR_ALIGNMENT"
    torch.cuda.synchronize()
    sccl.sccl_plan_destroy(pa)
    sccl.sccl_plan_destroy(pb)


@pytest.mark.parametrize("lowering", [M, S])
def test_one_plan_called_again_and_again(lowering):
    """A serving loop: the same plan on new data each time.  The library writes the table only when the array does
    not hold this plan's already, so the second and third call run on the table the first one left; a call for
    another plan in between replaces it, and the next call brings it back."""
    import torch
    sf = schedule_file.load("cfg5_allreduce_torus4x4")
    other = schedule_file.load("cfg2_allgather_hcm8")
    epc = 4 * 37
    plan = sccl.sccl_plan_create(*sf.descriptions("f32", epc), options={"flags": sccl.SCCL_PLAN_HOST_ONLY, "lowering": lowering})
    plan_b = sccl.sccl_plan_create(*other.descriptions("i32", 64), options={"flags": sccl.SCCL_PLAN_HOST_ONLY})
    hb = [inputs.generate("u32", "i32", 3, n, 0, other.positions_per_rank * 64) for n in range(8)]
    sched = Schedule(sf.rounds, sf.sends)
    print(f"[case] one plan again and again, lowering={lowering}", flush=True)
    for i, seed in enumerate((31, 32, 33, 34, 35)):
        if i == 3:                                         # another plan's table goes through the array
            db = [torch.from_numpy(h.copy()).cuda() for h in hb]
            sccl.sccl_execute_static(plan_b, db)
        host = [inputs.generate("wide", "f32", seed, n, 0, sf.num_chunks * epc) for n in range(16)]
        want = [h.copy() for h in host]
        ex.execute("f32", sf.num_chunks, epc, sched, want)
        got = [torch.from_numpy(h.copy()).cuda() for h in host]
        sccl.sccl_execute_static(plan, got)
        torch.cuda.synchronize()
        for n in range(16):
            assert (bits(got[n].cpu().numpy()) == bits(want[n])).all(), f"call {i}, rank {n}"
    sccl.sccl_plan_destroy(plan)
    sccl.sccl_plan_destroy(plan_b)


def test_large_slices_through_the_static_entry_point():
    """A host-only staged plan whose workgroups need 128 KiB of the local data share (more than a kernel gets without
    asking): the static entry point has to ask for it itself, since the plan's creation never touched the device."""
    import torch
    sf = schedule_file.load("cfg3_allreduce_hcm8")
    epc = 4 * (3 * 1024 + 17)
    host = [inputs.generate("wide", "f32", 211, n, 0, 8 * epc) for n in range(8)]
    want = [h.copy() for h in host]
    ex.execute("f32", 8, epc, Schedule(sf.rounds, sf.sends), want)
    plan = sccl.sccl_plan_create(*sf.descriptions("f32", epc), options={"flags": sccl.SCCL_PLAN_HOST_ONLY, "lowering": S,
                                                                         "slice_vectors": 1024})
    assert sccl.sccl_plan_stats(plan)["staged_lds_bytes"] > 64 * 1024
    got = [torch.from_numpy(h.copy()).cuda() for h in host]
    print("[case] static entry point, 128 KiB of local data share", flush=True)
    sccl.sccl_execute_static(plan, got)
    torch.cuda.synchronize()
    for n in range(8):
        assert (bits(got[n].cpu().numpy()) == bits(want[n])).all(), f"rank {n}"
    sccl.sccl_plan_destroy(plan)


@pytest.mark.parametrize("seed", list(range(100, 140)))
def test_random_cases_through_the_static_entry_point(seed):
    """Random topologies, collectives, element types and ragged sizes (tests/random_cases.py), one after the other
    through the one shared table, each under both lowerings with host-only plans: tables of every length follow each
    other in the static array."""
    from gpu_util import assert_same_bits, run_both
    from random_cases import random_case
    from test_random_schedules import make_inputs
    label, topo, coll, sched, dtype, dist, epc = random_case(seed)
    bufs = make_inputs(coll, dtype, dist, seed, epc)
    for lowering in (M, S):
        try:
            want, got = run_both(topo, coll, sched, dtype, bufs, epc, label=label, mode="sccl_execute_static",
                                 options={"lowering": lowering, "flags": sccl.SCCL_PLAN_HOST_ONLY})
        except sccl.ScclError as e:
            assert lowering == S and e.name == "SCCL_ERR_INVALID_ARG", (label, e.name)   # the cells do not fit the local data share
            continue
        assert_same_bits(want, got)


@pytest.mark.parametrize("lowering", [M, S])
def test_static_entry_point_under_graph_capture(lowering):
    """The table writes are kernels whose arguments hold the table words, so a captured call carries its own table:
    replays are right although another plan's table was written into the shared array in between."""
    import torch
    from gpu_util import assert_same_bits, host_inputs
    from helpers import to_binding
    from oracle import collective as col, generate as gen, topology as tp
    topo = tp.torus2d(4, 4)
    ag = col.allgather(16, 2)
    sched, coll = gen.compose_allreduce(gen.greedy_bfs(topo, ag), ag)
    P, G, epc = 16, coll.num_chunks, 4 * 1031
    plan = sccl.sccl_plan_create(*to_binding(topo, coll, sched, "f32", epc),
                                 options={"lowering": lowering, "flags": sccl.SCCL_PLAN_HOST_ONLY})
    small = schedule_file.load("cfg1_allgather_ring4")
    other = sccl.sccl_plan_create(*small.descriptions("i32", 700), options={"flags": sccl.SCCL_PLAN_HOST_ONLY})
    hb = [inputs.generate("u32", "i32", 8, n, 0, 4 * 700) for n in range(4)]
    db = [torch.from_numpy(h.copy()).cuda() for h in hb]
    pristine = [torch.zeros(G * epc, dtype=torch.float32, device="cuda") for _ in range(P)]
    work = [torch.empty_like(p) for p in pristine]
    print(f"[case] static entry point under graph capture, lowering={lowering}", flush=True)
    sccl.sccl_execute_static(other, db)                    # the first call on the device happens outside the capture
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        for w, p in zip(work, pristine):
            w.copy_(p)
        sccl.sccl_execute_static(plan, work, side)
    for seed in (5, 6, 7):
        bufs = host_inputs("wide", "f32", seed, P, G, epc)
        want = [b.copy() for b in bufs]
        ex.execute("f32", G, epc, sched, want)
        for p, b in zip(pristine, bufs):
            p.copy_(torch.from_numpy(b))
        sccl.sccl_execute_static(other, db)                # another table goes through the shared array
        torch.cuda.synchronize()
        print(f"[case]   replay seed={seed}", flush=True)
        graph.replay()
        torch.cuda.synchronize()
        assert_same_bits(want, [w.cpu().numpy() for w in work])
    for n in range(4):
        g = db[n].cpu().numpy()
        for c in range(4):
            assert (g[c * 700:(c + 1) * 700] == hb[c % 4][c * 700:(c + 1) * 700]).all()
    del graph
    sccl.sccl_plan_destroy(plan)
    sccl.sccl_plan_destroy(other)
