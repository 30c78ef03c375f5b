"""CPU tests of the library's host side: it loads, exports what include/sccl.h declares, and its
validation agrees with the oracle's verdict on good and bad plans (no kernel is launched here)."""
import ctypes
import os
import re

import numpy as np
import pytest

from helpers import VERDICT_TO_STATUS, plan_status
from oracle import collective as col
from oracle import executor as ex
from oracle import generate as gen
from oracle import topology as tp
from oracle.schedule import COPY, REDUCE, Schedule, make_schedule
from oracle.validate import validate
from paper_2008_08708_amd import sccl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "sccl.h")).read()
    declared = set(re.findall(r"\b(sccl_[a-z_]+)\s*\(", header))
    assert declared == set(sccl.EXPORTS)
    L = sccl.lib()
    for name in declared:
        assert getattr(L, name) is not None
    assert sccl.sccl_status_string(0) == "SCCL_OK"
    for i, name in enumerate(sccl.STATUS_NAMES):
        assert sccl.sccl_status_string(i) == name
        assert re.search(r"\b%s = %d\b" % (name, i), header)


def test_struct_layouts_match_the_header():
    # sizes a C compiler gives the structs of include/sccl.h on this ABI
    assert ctypes.sizeof(sccl.sccl_edge_t) == 8
    assert ctypes.sizeof(sccl.sccl_bw_t) == 16
    assert ctypes.sizeof(sccl.sccl_topology_t) == 24
    assert ctypes.sizeof(sccl.sccl_collective_t) == 56
    assert ctypes.sizeof(sccl.sccl_send_t) == 20
    assert ctypes.sizeof(sccl.sccl_schedule_t) == 32
    assert ctypes.sizeof(sccl.sccl_options_t) == 32


GOOD = [
    (tp.ring(4), 1, "greedy"), (tp.hcm8(), 1, "greedy"), (tp.hcm8(), 2, "greedy"), (tp.dgx1(), 2, "greedy"),
    (tp.torus2d(4, 4), 4, "greedy"), (tp.ring(8), 2, "ring"), (tp.ring(8), 4, "ring"), (tp.complete(5), 2, "greedy"),
]


@pytest.mark.parametrize("topo,C,kind", GOOD)
def test_valid_plans_are_accepted_and_counted_like_the_oracle(topo, C, kind):
    P = topo.num_nodes
    ag = col.allgather(P, C)
    s = gen.ring_allgather(P, C) if kind == "ring" else gen.greedy_bfs(topo, ag)
    ar, arc = gen.compose_allreduce(s, ag)
    rs, rsc = gen.reducescatter_from(s, ag)
    for (coll, sched, dtype, epc) in ((ag, s, "i32", 1000), (arc, ar, "f32", 1000), (rsc, rs, "f16", 1000)):
        assert validate(topo, coll, sched).ok
        name, st = plan_status(topo, coll, sched, dtype, epc)
        assert name == "SCCL_OK"
        cs = epc * (2 if dtype == "f16" else 4)
        fused, unfused = ex.algorithmic_bytes(sched, cs)
        assert (st["bytes_min"], st["bytes_unfused"]) == (fused, unfused)
        assert (st["num_steps"], st["num_rounds"], st["k"]) == (sched.num_steps, sched.num_rounds, sched.k)
        assert st["num_sends"] == sched.sends.shape[0]
        assert st["chunk_bytes"] == cs and st["bytes_per_rank"] == cs * coll.num_chunks


def test_headline_plan_statistics():
    ag = col.allgather(8, 1)
    ar, arc = gen.compose_allreduce(gen.greedy_bfs(tp.hcm8(), ag), ag)
    name, st = plan_status(tp.hcm8(), arc, ar, "f32", (32 << 20) // 4)
    assert name == "SCCL_OK"
    assert st["num_sends"] == 112 and st["num_steps"] == 4 and st["bytes_unfused"] == int(8.75 * 2 ** 30)
    assert st["bytes_per_rank"] == 256 << 20
    assert st["vector_bytes"] == 16 and st["num_work_items"] * st["block_threads"] * st["vectors_per_thread"] * 16 == 8 * (32 << 20)


def bad_plans():
    t3, ag3 = tp.ring(3), col.allgather(3, 1)
    good = [(n, n, (n + 1) % 3, 0) for n in range(3)] + [(n, n, (n - 1) % 3, 0) for n in range(3)]
    R, C = REDUCE, COPY
    ar3 = col.allreduce(3, 1)
    k4, bc4 = tp.complete(4), col.broadcast(4, 1, 0)
    yield t3, ag3, make_schedule([1], good)
    yield t3, ag3, make_schedule([1], [(3, 0, 1, 0)])
    yield t3, ag3, make_schedule([1], [(0, 0, 3, 0)])
    yield t3, ag3, make_schedule([1], [(0, 0, 1, 1)])
    yield t3, ag3, make_schedule([0], good)
    yield t3, ag3, make_schedule([1], [(0, 0, 0, 0)])
    yield t3, ag3, make_schedule([1], [(0, 0, 1, 0, 7)])
    yield t3, ag3, make_schedule([1], [(0, 0, 1, 0, R)])
    yield tp.ring(4), col.allgather(4, 1), make_schedule([1], [(0, 0, 2, 0)])
    yield t3, ag3, make_schedule([1], [(0, 1, 2, 0)])
    yield tp.ring(4), col.allgather(4, 1), make_schedule([1], [(0, 0, 1, 0), (0, 1, 2, 0)])
    yield t3, col.allgather(3, 2), make_schedule([1], [(0, 0, 1, 0), (3, 0, 1, 0)])
    yield t3, col.allgather(3, 2), make_schedule([2], [(0, 0, 1, 0), (3, 0, 1, 0)])
    yield t3, ag3, make_schedule([1], good[:-1])
    yield k4, bc4, make_schedule([1, 1], [(0, 0, 1, 0), (0, 0, 2, 0), (0, 1, 3, 1), (0, 2, 3, 1)])
    yield tp.shared_bus(3), ag3, make_schedule([1], good)
    yield tp.shared_bus(3), ag3, make_schedule([6], good)
    yield t3, ar3, make_schedule([1, 1, 1], [(0, 2, 1, 0, R), (0, 1, 0, 1, R), (0, 0, 1, 2, C), (0, 0, 2, 2, C)])
    yield t3, ar3, make_schedule([1, 1], [(0, 2, 1, 0, R), (0, 1, 0, 0, R), (0, 0, 1, 1, C), (0, 0, 2, 1, C)])
    yield t3, ar3, make_schedule([1, 1, 1], [(0, 2, 1, 0, R), (0, 2, 0, 0, R), (0, 1, 0, 1, R), (0, 0, 1, 2, C), (0, 0, 2, 2, C)])
    yield t3, ar3, make_schedule([1, 1, 1], [(0, 2, 1, 0, R), (0, 2, 0, 1, R), (0, 1, 0, 2, R)])
    yield t3, ar3, make_schedule([1, 1], [(0, 1, 0, 0, R), (0, 0, 1, 1, C), (0, 0, 2, 1, C)])
    yield t3, ar3, make_schedule([1], [(0, 1, 0, 0, C), (0, 2, 0, 0, R)])
    yield tp.ring(4), col.allgather(4, 1), gen.recursive_doubling_ring4()
    yield tp.ring(4), col.allgather(4, 1), Schedule([1, 1], gen.recursive_doubling_ring4().sends)
    # zero-bandwidth constraint blocks a link
    tz = tp.Topology(3, tuple(tp.ring(3).bw) + ((frozenset([(0, 1)]), 0),))
    yield tz, ag3, make_schedule([1], good)


@pytest.mark.parametrize("i,case", list(enumerate(bad_plans())))
def test_verdict_agrees_with_the_oracle(i, case):
    topo, coll, sched = case
    want = VERDICT_TO_STATUS[validate(topo, coll, sched).verdict.value]
    got, _ = plan_status(topo, coll, sched)
    assert got == want


def test_mutated_valid_schedules_get_the_same_verdict():
    # random single-field mutations of a valid Allreduce: the library and the oracle must agree on every one
    rng = np.random.default_rng(7)
    topo = tp.hcm8()
    ag = col.allgather(8, 1)
    ar, arc = gen.compose_allreduce(gen.greedy_bfs(topo, ag), ag)
    seen = set()
    for trial in range(300):
        sends = ar.sends.copy()
        i = rng.integers(0, sends.shape[0])
        f = rng.integers(0, 5)
        sends[i, f] = rng.integers(-1, 9) if f < 3 else (rng.integers(-1, 5) if f == 3 else rng.integers(0, 3))
        m = Schedule(list(ar.rounds), sends)
        want = VERDICT_TO_STATUS[validate(topo, arc, m).verdict.value]
        got, _ = plan_status(topo, arc, m)
        assert got == want, (i, f, sends[i])
        seen.add(got)
    assert len(seen) >= 5          # the mutations really exercise several error paths


def test_malformed_topology_and_arguments():
    t3, ag3 = tp.ring(3), col.allgather(3, 1)
    good = make_schedule([1], [(n, n, (n + 1) % 3, 0) for n in range(3)] + [(n, n, (n - 1) % 3, 0) for n in range(3)])
    bad_t = tp.Topology(3, ((frozenset([(0, 5)]), 1),))
    assert plan_status(bad_t, ag3, good)[0] == "SCCL_ERR_TOPOLOGY"
    bad_t = tp.Topology(3, ((frozenset([(1, 1)]), 1),))
    assert plan_status(bad_t, ag3, good)[0] == "SCCL_ERR_TOPOLOGY"
    bad_t = tp.Topology(3, ((frozenset([(0, 1)]), -1),))
    assert plan_status(bad_t, ag3, good)[0] == "SCCL_ERR_TOPOLOGY"
    assert plan_status(t3, ag3, good, options={"block_threads": 100})[0] == "SCCL_ERR_INVALID_ARG"
    assert plan_status(t3, ag3, good, options={"vectors_per_thread": 3})[0] == "SCCL_ERR_INVALID_ARG"
    assert plan_status(t3, ag3, good, elems_per_chunk=-1)[0] == "SCCL_ERR_INVALID_ARG"
    big = tp.ring(65)
    assert plan_status(big, col.allgather(65, 1), gen.greedy_bfs(big, col.allgather(65, 1)))[0] == "SCCL_ERR_INVALID_ARG"
    ok64 = tp.ring(64)
    assert plan_status(ok64, col.allgather(64, 1), gen.greedy_bfs(ok64, col.allgather(64, 1)))[0] == "SCCL_OK"


def test_execute_on_host_only_plan_is_refused():
    t3, ag3 = tp.ring(3), col.allgather(3, 1)
    good = make_schedule([1], [(n, n, (n + 1) % 3, 0) for n in range(3)] + [(n, n, (n - 1) % 3, 0) for n in range(3)])
    from helpers import to_binding
    p = sccl.sccl_plan_create(*to_binding(t3, ag3, good, "f32", 4), options={"flags": sccl.SCCL_PLAN_HOST_ONLY})
    with pytest.raises(sccl.ScclError) as e:
        sccl.sccl_execute(p, [16, 32, 48], stream=0)
    assert e.value.name == "SCCL_ERR_DEVICE"
    sccl.sccl_plan_destroy(p)


@pytest.mark.parametrize("dtype,epc,want_w", [("f32", 4, 16), ("f32", 6, 8), ("f32", 5, 4), ("f16", 8, 16), ("f16", 4, 8),
                                               ("f16", 2, 4), ("f16", 3, 2), ("i32", 1, 4), ("f32", 0, 16)])
def test_vector_width_follows_the_chunk_size(dtype, epc, want_w):
    t3, ag3 = tp.ring(3), col.allgather(3, 1)
    good = make_schedule([1], [(n, n, (n + 1) % 3, 0) for n in range(3)] + [(n, n, (n - 1) % 3, 0) for n in range(3)])
    name, st = plan_status(t3, ag3, good, dtype, epc)
    assert name == "SCCL_OK" and st["vector_bytes"] == want_w


def test_work_distribution_follows_chunk_size_and_fan_in():
    topo = tp.torus2d(4, 4)
    ag = col.allgather(16, 4)
    s = gen.greedy_bfs(topo, ag)
    _, tiny = plan_status(topo, ag, s, "f32", 4)                 # 16-byte chunks: one vector each
    assert (tiny["block_threads"], tiny["vectors_per_thread"], tiny["num_work_items"]) == (64, 1, 64)
    _, big = plan_status(topo, ag, s, "f32", (16 << 20) // 4)     # copy only: 8 vectors per lane
    assert (big["block_threads"], big["vectors_per_thread"]) == (256, 8)
    assert big["num_work_items"] == 64 * ((16 << 20) // (256 * 8 * 16))
    # the headline Allreduce has fan-in 4: five loads per vector, so four vectors per lane
    ag8 = col.allgather(8, 1)
    ar, arc = gen.compose_allreduce(gen.greedy_bfs(tp.hcm8(), ag8), ag8)
    _, head = plan_status(tp.hcm8(), arc, ar, "f32", (32 << 20) // 4)
    assert head["max_fan_in"] == 4 and (head["block_threads"], head["vectors_per_thread"]) == (256, 4)
    # a ring has fan-in 1
    rar, rarc = gen.compose_allreduce(gen.ring_allgather(8, 4), col.allgather(8, 4))
    _, ring = plan_status(tp.ring(8), rarc, rar, "f16", (16 << 20) // 2)
    assert ring["max_fan_in"] == 1 and ring["vectors_per_thread"] == 8
    # a copy chain (each forwarded chunk is read back by the very next write) takes 16 KiB tiles, which the L2 still
    # holds at the next hop; with any other write in between, or a fan-out, it is 8 vectors again
    _, chain = plan_status(tp.ring(8), col.allgather(8, 2), gen.ring_allgather(8, 2), "f32", (4 << 20) // 4)
    assert (chain["max_fan_out"], chain["block_threads"], chain["vectors_per_thread"]) == (1, 256, 4)
    for make in (lambda: col.gather(8, 2, 0), lambda: col.alltoall(8, 8)):
        c = make()
        _, st = plan_status(tp.ring(8), c, gen.greedy_route(tp.ring(8), c), "f32", (1 << 20) // 4)
        assert st["vectors_per_thread"] == 4, c.name
    bc = col.broadcast(8, 4, 0)                                   # both directions interleave: the distance is 2
    _, far = plan_status(tp.ring(8), bc, gen.greedy_route(tp.ring(8), bc), "f32", (16 << 20) // 4)
    assert (far["max_fan_out"], far["vectors_per_thread"]) == (1, 8)
    sc = col.scatter(8, 2, 0)
    direct = gen.greedy_route(tp.complete(8), sc)                 # one hop: nothing is read back
    _, st = plan_status(tp.complete(8), sc, direct, "f32", (4 << 20) // 4)
    assert st["max_chunk_groups"] == 1 and st["vectors_per_thread"] == 8
    # every choice still tiles the chunk exactly
    for st in (tiny, big, head, ring, chain, far):
        tile = st["block_threads"] * st["vectors_per_thread"] * st["vector_bytes"]
        assert st["num_work_items"] == st["num_global_chunks"] * -(-st["chunk_bytes"] // tile)


def test_other_collectives_are_accepted():
    for topo in (tp.ring(8), tp.hcm8(), tp.torus2d(4, 4)):
        P = topo.num_nodes
        for coll in (col.broadcast(P, 3, 1), col.gather(P, 2, P - 1), col.scatter(P, 2 * P, 0), col.alltoall(P, P)):
            s = gen.greedy_route(topo, coll)
            assert validate(topo, coll, s).ok
            name, st = plan_status(topo, coll, s, "f32", 64)
            assert name == "SCCL_OK" and st["num_reduce_groups"] == 0
            assert st["bytes_min"] == ex.algorithmic_bytes(s, 256)[0]
        bc = col.broadcast(P, 2, 0)
        red = gen.invert(gen.greedy_route(topo, bc), bc)
        name, st = plan_status(topo.reversed(), col.reduce(P, 2, 0), red, "f16", 64)
        assert name == "SCCL_OK" and st["num_copy_groups"] == 0


def test_slot_maps_are_validated():
    topo, coll = tp.ring(4), col.alltoall(4, 4)
    s = gen.greedy_route(topo, coll)
    slot, per_rank = col.compact_slots(coll, s.sends)
    assert per_rank < coll.num_chunks                       # the point of a compact layout
    name, st = plan_status(topo, coll, s, "f32", 8, slot=slot, slots_per_rank=per_rank)
    assert name == "SCCL_OK" and st["bytes_per_rank"] == per_rank * 32
    # a chunk in pre without a position
    bad = slot.copy(); bad[0, 0] = -1
    assert plan_status(topo, coll, s, "f32", 8, slot=bad, slots_per_rank=per_rank)[0] == "SCCL_ERR_INVALID_ARG"
    # a destination of a send without a position
    c, n, m = s.sends[0, 0], s.sends[0, 1], s.sends[0, 2]
    bad = slot.copy(); bad[c, m] = -1
    assert plan_status(topo, coll, s, "f32", 8, slot=bad, slots_per_rank=per_rank)[0] == "SCCL_ERR_INVALID_ARG"
    # two chunks in one position of one rank
    bad = slot.copy()
    held = np.nonzero(bad[:, 0] >= 0)[0]
    bad[held[1], 0] = bad[held[0], 0]
    assert plan_status(topo, coll, s, "f32", 8, slot=bad, slots_per_rank=per_rank)[0] == "SCCL_ERR_INVALID_ARG"
    # out of range position, empty buffer
    bad = slot.copy(); bad[held[0], 0] = per_rank
    assert plan_status(topo, coll, s, "f32", 8, slot=bad, slots_per_rank=per_rank)[0] == "SCCL_ERR_INVALID_ARG"
    assert plan_status(topo, coll, s, "f32", 8, slot=slot, slots_per_rank=0)[0] == "SCCL_ERR_INVALID_ARG"


# ---- the staged lowering: dependency levels and cells are host logic, checked here without a GPU

def _levels_by_hand(sched):
    """Longest chain of dependent groups, from the definition: a group depends on an earlier group if it reads a
    cell that group wrote, or writes a cell that group read or wrote."""
    from collections import OrderedDict
    groups = []
    for s in range(sched.num_steps):
        gs = OrderedDict()
        for (c, n, m, st, op) in sched.sends.tolist():
            if st != s:
                continue
            if op == COPY:
                gs.setdefault((0, c, n), []).append(m)
            else:
                gs.setdefault((1, c, m), []).append(n)
        for (kind, c, a), others in gs.items():
            reads = {(c, a)} | ({(c, o) for o in others} if kind == 1 else set())
            writes = {(c, a)} if kind == 1 else {(c, o) for o in others}
            groups.append((reads, writes))
    depth = []
    for i, (r, w) in enumerate(groups):
        d = 1
        for j in range(i):
            rj, wj = groups[j]
            if (r & wj) or (w & rj) or (w & wj):
                d = max(d, depth[j] + 1)
        depth.append(d)
    cells = set().union(*[r | w for r, w in groups])
    written = set().union(*[w for _, w in groups])
    first_read = set()
    seen = set()
    for r, w in groups:
        first_read |= (r - seen)
        seen |= r | w
    return max(depth), len(cells), len(first_read), len(written)


@pytest.mark.parametrize("topo,C,kind", GOOD)
def test_staged_tables_follow_the_dependency_structure(topo, C, kind):
    P = topo.num_nodes
    ag = col.allgather(P, C)
    s = gen.ring_allgather(P, C) if kind == "ring" else gen.greedy_bfs(topo, ag)
    ar, arc = gen.compose_allreduce(s, ag)
    for coll, sched in ((ag, s), (arc, ar)):
        name, st = plan_status(topo, coll, sched, "f32", 4)
        assert name == "SCCL_OK" and st["staged_available"] == 1
        levels, cells, loaded, stored = _levels_by_hand(sched)
        assert (st["num_levels"], st["num_cells"], st["num_cells_loaded"], st["num_cells_stored"]) == (levels, cells, loaded, stored)
        assert st["num_levels"] <= sched.num_steps
        assert st["lowering"] == sccl.SCCL_LOWER_STAGED           # 16 bytes per chunk: small


def test_staged_lowering_choice_and_limits():
    topo, ag = tp.torus2d(4, 4), col.allgather(16, 4)
    s = gen.greedy_bfs(topo, ag)
    ar, arc = gen.compose_allreduce(s, ag)
    # torus Allgather: every chunk reaches 15 ranks over a tree of depth <= diameter + waiting; Allreduce twice that
    _, st = plan_status(topo, ag, s, "f32", 4)
    assert st["num_cells"] == 16 * 64 and st["num_cells_loaded"] == 64 and st["num_cells_stored"] == 15 * 64
    _, st2 = plan_status(topo, arc, ar, "f32", 4)
    assert st2["num_cells_loaded"] == 16 * 64 and st2["num_levels"] == 2 * st["num_levels"]
    # auto: staged up to 16 MiB over all ranks, through memory above
    for epc, want in ((1 << 12, sccl.SCCL_LOWER_STAGED), (1 << 13, sccl.SCCL_LOWER_MEMORY)):
        _, st = plan_status(topo, arc, ar, "f32", epc)
        assert P_bytes(st) == 16 * 64 * epc * 4 and st["lowering"] == want
    # a ring Allreduce saves 7 of its 14 round trips per chunk: staged while the work items are few (4096), by size beyond
    ring, rag = tp.ring(8), col.allgather(8, 4)
    rar, rarc = gen.compose_allreduce(gen.ring_allgather(8, 4), rag)
    for epc, want in ((512, sccl.SCCL_LOWER_STAGED), (8192, sccl.SCCL_LOWER_STAGED), (16384, sccl.SCCL_LOWER_MEMORY)):
        _, st = plan_status(ring, rarc, rar, "f32", epc)                                    # 32 chunks x epc / 4 / 16 work items
        assert st["lowering"] == want and st["max_chunk_groups"] == st["num_levels"] == 14 and st["staged_levels"] == 7
    # two-hop schedules save too little: staged only while tiny (512 KiB over all ranks)
    g8, gc = tp.dgx1(), col.gather(8, 1, 0)
    gs = gen.greedy_route(g8, gc)
    for epc, want in ((2048, sccl.SCCL_LOWER_STAGED), (4096, sccl.SCCL_LOWER_MEMORY)):      # 8 chunks x 8 ranks x epc x 4 B
        assert plan_status(g8, gc, gs, "f32", epc)[1]["lowering"] == want
    k8, kag = tp.complete(8), col.allgather(8, 1)
    kar, karc = gen.compose_allreduce(gen.greedy_bfs(k8, kag), kag)
    assert plan_status(k8, karc, kar, "f32", 1 << 16)[1]["lowering"] == sccl.SCCL_LOWER_MEMORY       # 2 groups per chunk
    # explicit choices
    st = plan_status(topo, arc, ar, "f32", 1 << 14, options={"lowering": sccl.SCCL_LOWER_STAGED})[1]
    assert st["lowering"] == sccl.SCCL_LOWER_STAGED and st["slice_vectors"] == 16 and st["staged_threads"] == 64
    st = plan_status(topo, arc, ar, "f32", 16)[1]          # 4 vectors per chunk, 64 chunks: one vector per work item
    assert st["slice_vectors"] == 1 and st["num_slices"] == 256
    assert plan_status(topo, arc, ar, "f32", 4, options={"lowering": sccl.SCCL_LOWER_MEMORY})[1]["lowering"] == sccl.SCCL_LOWER_MEMORY
    # a slice of every cell of a chunk (16 ranks hold it) must fit 160 KiB together with the chunk's tables
    assert plan_status(topo, arc, ar, "f32", 1 << 12, options={"lowering": sccl.SCCL_LOWER_STAGED, "slice_vectors": 1024})[0] == "SCCL_ERR_INVALID_ARG"
    _, st = plan_status(topo, arc, ar, "f32", 1 << 12, options={"lowering": sccl.SCCL_LOWER_STAGED, "slice_vectors": 512})
    assert st["slice_vectors"] == 512 and st["num_slices"] == 64 * 2 and 128 * 1024 < st["staged_lds_bytes"] <= 160 * 1024
    _, st = plan_status(topo, arc, ar, "f32", 1 << 10, options={"lowering": sccl.SCCL_LOWER_STAGED, "slice_vectors": 4})
    assert st["slice_vectors"] == 4 and st["num_slices"] == 64 * 64
    for bad in ({"lowering": 3}, {"slice_vectors": 3}, {"staged_threads": 96}, {"reserved": 1}):
        assert plan_status(topo, arc, ar, "f32", 4, options=bad)[0] == "SCCL_ERR_INVALID_ARG"


def P_bytes(st):
    return st["num_nodes"] * st["bytes_per_rank"]


def test_hostile_sizes_and_enum_values_are_refused_not_trusted():
    topo, ag = tp.ring(4), col.allgather(4, 1)
    s = gen.greedy_bfs(topo, ag)
    # element counts whose byte sizes do not fit 63 bits (chunk, rank buffer or the statistics' byte counts)
    for epc in ((1 << 62) + 5, (1 << 63) - 1, 1 << 61):
        assert plan_status(topo, ag, s, "f32", epc)[0] == "SCCL_ERR_INVALID_ARG"
    assert plan_status(topo, ag, s, "f32", -1)[0] == "SCCL_ERR_INVALID_ARG"
    name, st = plan_status(topo, ag, s, "f16", 1 << 40, options={"lowering": sccl.SCCL_LOWER_MEMORY})
    assert name == "SCCL_OK" and st["bytes_per_rank"] == 4 * 2 * (1 << 40)      # large but representable
    # an integer that is no sccl_dtype_t in the enum's place
    sccl.DTYPE_CODES["not-a-dtype"] = 256
    try:
        assert plan_status(topo, ag, s, "not-a-dtype", 4)[0] == "SCCL_ERR_INVALID_ARG"
    finally:
        del sccl.DTYPE_CODES["not-a-dtype"]


def test_static_table_size_is_reported_and_oversized_plans_are_refused_without_a_device():
    """sccl_execute_static places the step table in a static device array of SCCL_STATIC_SCRATCH_BYTES: the
    size check comes before any device call, so it can be seen here."""
    import ctypes as ct
    topo, ag = tp.ring(4), col.allgather(4, 1)
    s = gen.greedy_bfs(topo, ag)
    p = sccl.sccl_plan_create(*__import__("helpers").to_binding(topo, ag, s, "f32", 64),
                              options={"flags": sccl.SCCL_PLAN_HOST_ONLY, "lowering": sccl.SCCL_LOWER_MEMORY})
    st = sccl.sccl_plan_stats(p)
    # chunk offsets (G + 1 words, padded to 4), then header + anchor + others per group
    groups = st["num_copy_groups"] + st["num_reduce_groups"]
    assert st["static_table_bytes"] == 4 * (8 + 2 * groups + st["num_sends"])
    sccl.sccl_plan_destroy(p)
    # a ring Allgather on 64 ranks with 24 chunks per node: 96 768 sends, a table of about 1 MiB
    topo, ag = tp.ring(64), col.allgather(64, 24)
    s = gen.ring_allgather(64, 24)
    p = sccl.sccl_plan_create(*__import__("helpers").to_binding(topo, ag, s, "f32", 4),
                              options={"flags": sccl.SCCL_PLAN_HOST_ONLY, "lowering": sccl.SCCL_LOWER_MEMORY})
    assert sccl.sccl_plan_stats(p)["static_table_bytes"] > sccl.SCCL_STATIC_SCRATCH_BYTES
    fake = [0x1000 * (n + 1) for n in range(64)]           # never dereferenced: the call must fail before any launch
    with pytest.raises(sccl.ScclError) as e:
        sccl.sccl_execute_static(p, fake, stream=0)
    assert e.value.name == "SCCL_ERR_SCRATCH"
    with pytest.raises(ValueError):
        sccl.sccl_execute_static(p, fake[:3], stream=0)
    sccl.sccl_plan_destroy(p)


def awkward_copy_schedules():
    """Valid combining schedules on three fully connected ranks in which a COPY cannot be propagated by the staged
    lowering: its source (first) or its destination (second) is written again afterwards."""
    from oracle.collective import Collective
    topo = tp.complete(3)
    pre = np.ones((1, 3), dtype=np.uint8)
    for last, root in (((0, 2, 0, 2, REDUCE), 0), ((0, 2, 1, 2, REDUCE), 1)):
        post = np.zeros((1, 3), dtype=np.uint8)
        post[0, root] = 1
        coll = Collective("reduce-with-a-detour", 3, 1, pre, post, True)
        sched = make_schedule([1, 1, 1], [(0, 1, 0, 0, REDUCE), (0, 0, 1, 1, COPY), last])
        yield topo, coll, sched


def test_copy_propagation_of_the_staged_lowering():
    # non-combining collectives: every copy's source stays put, so no level and no task is left
    for topo, coll in ((tp.torus2d(4, 4), col.allgather(16, 4)), (tp.dgx1(), col.alltoall(8, 8)), (tp.hcm8(), col.broadcast(8, 3, 1))):
        s = gen.greedy_route(topo, coll) if coll.name != "allgather" else gen.greedy_bfs(topo, coll)
        _, st = plan_status(topo, coll, s, "f32", 64)
        assert st["num_levels"] >= 2 and st["staged_levels"] == 0 and st["staged_tasks"] == 0
    # Allreduce = Reducescatter ; Allgather: the reducing half keeps its levels, the copying half has none
    for topo, C, kind in ((tp.torus2d(4, 4), 4, "greedy"), (tp.ring(8), 2, "ring"), (tp.hcm8(), 1, "greedy")):
        ag = col.allgather(topo.num_nodes, C)
        base = gen.ring_allgather(8, C) if kind == "ring" else gen.greedy_bfs(topo, ag)
        ar, arc = gen.compose_allreduce(base, ag)
        rs, rsc = gen.reducescatter_from(base, ag)
        _, st = plan_status(topo, arc, ar, "f32", 64)
        _, st_rs = plan_status(topo.reversed(), rsc, rs, "f32", 64)
        assert st["staged_levels"] == st_rs["staged_levels"] == st_rs["num_levels"] == st["num_levels"] // 2
        assert st["staged_tasks"] == st_rs["staged_tasks"] == st["num_reduce_groups"]
    # copies whose source or destination is written again stay tasks
    for topo, coll, sched in awkward_copy_schedules():
        assert validate(topo, coll, sched).ok
        _, st = plan_status(topo, coll, sched, "f32", 64)
        assert st["staged_tasks"] == 3 and st["staged_levels"] == st["num_levels"] == 3
