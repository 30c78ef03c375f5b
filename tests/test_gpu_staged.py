"""GPU parity of the staged lowering (a chunk's sends run in the local data share): launch shapes, slice sizes,
ragged last slices, every vector width, several slices per workgroup, slot maps.  The other GPU tests already run
every case under both lowerings (gpu_util.run_both); these pin what is specific to this one."""
import numpy as np
import pytest

from gpu_util import assert_same_bits, bits, host_inputs, run_both
from helpers import to_binding
from oracle import collective as col
from oracle import generate as gen
from oracle import topology as tp
from paper_2008_08708_amd import sccl

pytestmark = pytest.mark.gpu
STAGED = sccl.SCCL_LOWER_STAGED


def case(topo, C, what, kind="greedy"):
    P = topo.num_nodes
    ag = col.allgather(P, C)
    base = gen.ring_allgather(P, C) if kind == "ring" else gen.greedy_bfs(topo, ag)
    if what == "allgather":
        return ag, base, ag.pre
    sched, coll = gen.compose_allreduce(base, ag)
    return coll, sched, None


@pytest.mark.parametrize("slice_vectors", [1, 2, 8, 32])
@pytest.mark.parametrize("threads", [64, 256, 1024])
@pytest.mark.parametrize("what,dtype,dist", [("allreduce", "f32", "uniform"), ("allgather", "i32", "u32"), ("allreduce", "f16", "normal")])
def test_slices_and_workgroup_sizes(slice_vectors, threads, what, dtype, dist):
    topo = tp.hcm8()
    coll, sched, pre = case(topo, 2, what)
    # 37 whole vectors per chunk plus nothing ragged at the vector level: slices of 2, 8 and 32 end ragged
    epc = 37 * (4 if dtype != "f16" else 8)
    bufs = host_inputs(dist, dtype, 83, 8, coll.num_chunks, epc, pre)
    want, got = run_both(topo, coll, sched, dtype, bufs, epc, label=f"staged-{what}",
                         options={"lowering": STAGED, "slice_vectors": slice_vectors, "staged_threads": threads})
    assert_same_bits(want, got)


@pytest.mark.parametrize("epc,dtype", [(1, "f32"), (3, "f32"), (6, "f32"), (1, "f16"), (2, "f16"), (4, "f16"), (1036, "f16"), (1031, "i32")])
def test_every_vector_width(epc, dtype):
    topo = tp.torus2d(4, 4)
    coll, sched, _ = case(topo, 1, "allreduce")
    dist = {"f32": "uniform", "f16": "normal", "i32": "u32"}[dtype]
    bufs = host_inputs(dist, dtype, 89, 16, coll.num_chunks, epc)
    want, got = run_both(topo, coll, sched, dtype, bufs, epc, label=f"staged-width-{epc}-{dtype}", options={"lowering": STAGED})
    assert_same_bits(want, got)


@pytest.mark.parametrize("grid", [1, 3])
def test_one_workgroup_walks_every_slice(grid):
    topo = tp.torus2d(4, 4)
    coll, sched, _ = case(topo, 4, "allreduce")
    epc = 4 * 21 + 4                                      # 22 vectors per chunk: 11 slices of 2, or 22 of 1, per chunk
    bufs = host_inputs("uniform", "f32", 97, 16, coll.num_chunks, epc)
    for sv in (1, 2):
        want, got = run_both(topo, coll, sched, "f32", bufs, epc, label=f"staged-grid{grid}",
                             options={"lowering": STAGED, "slice_vectors": sv, "max_workgroups": grid})
        assert_same_bits(want, got)


def test_config5_smallest_sizes_are_staged_by_default():
    topo = tp.torus2d(4, 4)
    for what in ("allgather", "allreduce"):
        coll, sched, pre = case(topo, 4, what)
        for epc in (4, 16, 64):
            plan = sccl.sccl_plan_create(*to_binding(topo, coll, sched, "f32", epc))
            st = sccl.sccl_plan_stats(plan)
            sccl.sccl_plan_destroy(plan)
            assert st["lowering"] == STAGED and st["staged_lds_bytes"] <= 160 * 1024
            bufs = host_inputs("uniform", "f32", 101, 16, coll.num_chunks, epc, pre)
            want, got = run_both(topo, coll, sched, "f32", bufs, epc, label=f"staged-cfg5-{what}-{epc}", options={"lowering": 0})
            assert_same_bits(want, got)


def test_large_slices_use_the_whole_local_data_share():
    # 8 cells per chunk x 1024 vectors x 16 B = 128 KiB of cells: more than the 64 KiB a kernel gets without asking
    topo = tp.hcm8()
    coll, sched, _ = case(topo, 1, "allreduce")
    epc = 4 * (3 * 1024 + 17)
    bufs = host_inputs("uniform", "f32", 103, 8, coll.num_chunks, epc)
    want, got = run_both(topo, coll, sched, "f32", bufs, epc, label="staged-128KiB",
                         options={"lowering": STAGED, "slice_vectors": 1024})
    assert_same_bits(want, got)
    for g in got[1:]:
        assert (bits(g) == bits(got[0])).all()


def test_repeated_execution_reuses_the_plan():
    import torch
    topo = tp.ring(8)
    coll, sched, _ = case(topo, 2, "allreduce", kind="ring")
    epc = 8 * 9
    plan = sccl.sccl_plan_create(*to_binding(topo, coll, sched, "i32", epc), options={"lowering": STAGED})
    from oracle import executor as ex
    for seed in (1, 2, 3):
        bufs = host_inputs("u32", "i32", seed, 8, coll.num_chunks, epc)
        want = [b.copy() for b in bufs]
        ex.execute("i32", coll.num_chunks, epc, sched, want)
        dev = [torch.from_numpy(b.copy()).cuda() for b in bufs]
        print(f"[case] staged plan reuse seed={seed}", flush=True)
        sccl.sccl_execute(plan, dev)
        torch.cuda.synchronize()
        assert_same_bits(want, [d.cpu().numpy() for d in dev])
    sccl.sccl_plan_destroy(plan)


def test_copies_that_cannot_be_propagated_stay_tasks():
    # the staged lowering stores the destination of a COPY from the source's place in the local data share unless
    # source or destination is written again: these schedules do exactly that (and leave a partial sum behind)
    from test_host_plan import awkward_copy_schedules
    for i, (topo, coll, sched) in enumerate(awkward_copy_schedules()):
        for dtype, dist in (("f32", "uniform"), ("f16", "normal"), ("i32", "u32")):
            epc = 4 * 37 + 4
            bufs = host_inputs(dist, dtype, 107 + i, 3, 1, epc)
            want, got = run_both(topo, coll, sched, dtype, bufs, epc, label=f"awkward-copy-{i}-{dtype}")
            assert_same_bits(want, got)
