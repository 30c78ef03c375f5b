"""The plan compiler without a GPU: the step tables sccl_plan_create emits (sccl_plan_table) are INTERPRETED here in
numpy, word by word as include/sccl.h documents them and as the kernels walk them, and the buffers that leaves are
compared bit for bit with the oracle's.  This covers, on the CPU, everything between a validated schedule and the
kernel's inner loop: grouping, operand encoding, slot maps, the staged lowering's cells, copy propagation, levels,
identity slots and overflow sources.  (That the kernels interpret the tables the same way is what the GPU tests show.)
"""
import numpy as np
import pytest

from helpers import to_binding
from oracle import collective as col
from oracle import executor as ex
from oracle import generate as gen
from oracle import topology as tp
from oracle.schedule import COPY, REDUCE, make_schedule
from paper_2008_08708_amd import inputs, schedule_file, sccl
from random_cases import random_case

NP = {"i32": np.int32, "f32": np.float32, "f16": np.float16}
HOST = sccl.SCCL_PLAN_HOST_ONLY


def add(acc, x, dtype):
    """acc + x the way both sides do it: wrapping int32, or IEEE binary32 (binary16 operands are widened exactly)."""
    if dtype == "i32":
        return (acc.view(np.uint32) + x.view(np.uint32)).view(np.int32)
    return (acc.astype(np.float32) + x.astype(np.float32)).astype(np.float32)


def chunk_of(bufs, operand, epc):
    rank, pos = operand & 0xff, operand >> 8
    return bufs[rank][pos * epc:(pos + 1) * epc]


def interpret_memory_table(words, info, G, dtype, epc, bufs):
    prog = info[0]
    for c in range(G):
        w, end = prog + words[c], prog + words[c + 1]
        while w < end:
            hdr, anchor = int(words[w]), int(words[w + 1])
            k = hdr >> 8
            others = [int(x) for x in words[w + 2:w + 2 + k]]
            if hdr & 1:
                acc = chunk_of(bufs, anchor, epc).astype(np.float32 if dtype != "i32" else np.int32)
                for o in others:
                    acc = add(acc, chunk_of(bufs, o, epc), dtype)
                chunk_of(bufs, anchor, epc)[:] = acc.astype(NP[dtype])          # one narrowing per group
            else:
                src = chunk_of(bufs, anchor, epc).copy()
                for o in others:
                    chunk_of(bufs, o, epc)[:] = src
            w += 2 + k
        assert w == end


def interpret_staged_table(words, info, G, dtype, epc, bufs, vector_bytes):
    block_words, room, log_slice, identity = info
    elems_per_vector = vector_bytes // NP[dtype]().itemsize
    slice_elems = (1 << log_slice) * elems_per_vector
    slice_bytes = (1 << log_slice) * vector_bytes
    ident = {"i32": np.int32(0), "f32": np.float32(-0.0), "f16": np.float16(-0.0)}[dtype]
    for c in range(G):
        b = words[c * block_words:(c + 1) * block_words]
        n_store, n_in, n_out, n_levels, n_tasks, n_extra = (int(x) for x in b[:6])
        assert n_in <= n_store <= room and identity == room_to_identity(words, info, G, slice_bytes)
        lev = 8 + room
        out = lev + n_levels + 2
        task = (out + 2 * n_out + 3) & ~3
        extra = task + 8 * n_tasks
        assert extra + n_extra <= block_words
        firsts = [int(x) for x in b[lev:lev + n_levels + 2]]
        assert firsts[0] == 0 and firsts[n_levels] == firsts[n_levels + 1] == n_tasks and firsts == sorted(firsts)
        for s0 in range(0, epc, slice_elems):                                    # one work item per slice
            n = min(slice_elems, epc - s0)
            lds = {}                                                             # storage byte offset -> slice
            for i in range(n_in):
                lds[i * slice_bytes] = chunk_of(bufs, int(b[8 + i]), epc)[s0:s0 + n].copy()
            lds[identity] = np.full(n, ident, dtype=NP[dtype])
            for lv in range(n_levels):
                writes = {}
                for t in range(firsts[lv], firsts[lv + 1]):
                    rec = [int(x) for x in b[task + 8 * t:task + 8 * t + 8]]
                    dst, k = rec[0] & 0xffffff, rec[0] >> 24
                    assert dst % slice_bytes == 0 and dst not in writes and rec[6] == rec[7] == 0
                    if k == 0:
                        writes[dst] = lds[rec[2]].copy()
                        continue
                    acc = lds[dst].astype(np.float32 if dtype != "i32" else np.int32)
                    for j in range(4):
                        assert rec[2 + j] == identity or j < k
                        acc = add(acc, lds[rec[2 + j]], dtype)
                    for j in range(4, k):
                        acc = add(acc, lds[int(b[extra + rec[1] + j - 4])], dtype)
                    writes[dst] = acc.astype(NP[dtype])
                lds.update(writes)                                               # a level's tasks see the level's start
            for i in range(n_out):
                chunk_of(bufs, int(b[out + 2 * i + 1]), epc)[s0:s0 + n] = lds[int(b[out + 2 * i])]


def room_to_identity(words, info, G, slice_bytes):
    most = max(int(words[c * info[0]]) for c in range(G))                        # storages of the fullest chunk
    return most * slice_bytes


def check(topo, coll, sched, dtype, dist, epc, seed=5, slot=None, slots_per_rank=0, options=None):
    P, G = coll.num_nodes, coll.num_chunks
    K = slots_per_rank if slot is not None else G
    bufs = [inputs.generate(dist, dtype, seed, n, 0, K * epc) for n in range(P)]
    if not coll.combining:
        for n in range(P):
            held = {int(c if slot is None else slot[c, n]) for c in range(G) if coll.pre[c, n]}
            for k in range(K):
                if k not in held:
                    inputs.poison(bufs[n], k * epc, (k + 1) * epc)
    want = [b.copy() for b in bufs]
    ex.execute(dtype, G, epc, sched, want, slot=slot, slots_per_rank=slots_per_rank if slot is not None else None)
    opts = {"flags": HOST}
    opts.update(options or {})
    plan = sccl.sccl_plan_create(*to_binding(topo, coll, sched, dtype, epc, slot, slots_per_rank), options=opts)
    st = sccl.sccl_plan_stats(plan)
    u = np.uint32 if dtype != "f16" else np.uint16
    words, info = sccl.sccl_plan_table(plan, sccl.SCCL_LOWER_MEMORY)
    got = [b.copy() for b in bufs]
    interpret_memory_table(words, info, G, dtype, epc, got)
    for n in range(P):
        assert (got[n].view(u) == want[n].view(u)).all(), f"through-memory table, rank {n}"
    assert st["static_table_bytes"] == 4 * len(words) or st["lowering"] == sccl.SCCL_LOWER_STAGED
    if st["staged_available"]:
        words, info = sccl.sccl_plan_table(plan, sccl.SCCL_LOWER_STAGED)
        got = [b.copy() for b in bufs]
        interpret_staged_table(words, info, G, dtype, epc, got, st["vector_bytes"])
        for n in range(P):
            assert (got[n].view(u) == want[n].view(u)).all(), f"staged table, rank {n}"
    else:
        with pytest.raises(sccl.ScclError):
            sccl.sccl_plan_table(plan, sccl.SCCL_LOWER_STAGED)
    sccl.sccl_plan_destroy(plan)
    return st


SCHEDULES = ["cfg1_allgather_ring4", "cfg2_allgather_hcm8", "cfg3_allreduce_hcm8", "cfg4_allreduce_ring8", "cfg5_allgather_torus4x4",
             "cfg5_allreduce_torus4x4", "cfg5_allreduce_torus4x4_latency", "alltoall_dgx1", "broadcast_dgx1", "reduce_dgx1",
             "gather_dgx1", "scatter_dgx1", "reducescatter_dgx1"]


@pytest.mark.parametrize("name", SCHEDULES)
@pytest.mark.parametrize("dtype,dist,epc", [("f32", "uniform", 4 * 37), ("f16", "normal", 8 * 5 + 2), ("i32", "u32", 9)])
def test_stored_schedules_through_both_tables(name, dtype, dist, epc):
    sf = schedule_file.load(name)
    topo, coll, sched = sf.descriptions(dtype, epc)
    # the binding's descriptions carry what the oracle-side helpers need under other names
    from oracle.collective import Collective
    from oracle.schedule import Schedule
    from oracle.topology import Topology
    otopo = Topology(sf.num_nodes, tuple((frozenset(L), b) for L, b in sf.bw), name)
    ocoll = Collective(sf.collective, sf.num_nodes, sf.num_chunks, sf.pre, sf.post, sf.combining)
    st = check(otopo, ocoll, Schedule(sf.rounds, sf.sends), dtype, dist, epc, slot=sf.slot, slots_per_rank=sf.slots_per_rank)
    assert st["staged_available"] == 1


@pytest.mark.parametrize("slice_vectors", [1, 2, 8])
def test_slices_ragged_tails_and_fan_in_above_four(slice_vectors):
    # a complete graph of 8: one step reduces 7 sources into each root (three overflow sources per task)
    topo, ag = tp.complete(8), col.allgather(8, 1)
    ar, arc = gen.compose_allreduce(gen.greedy_bfs(topo, ag), ag)
    st = check(topo, arc, ar, "f32", "uniform", 4 * 11 + 1, options={"slice_vectors": slice_vectors})
    assert st["max_fan_in"] == 7
    st = check(topo, arc, ar, "f16", "normal", 8 * 3 + 4, options={"slice_vectors": slice_vectors})
    check(tp.torus2d(4, 4), *reversed(gen.compose_allreduce(gen.greedy_bfs(tp.torus2d(4, 4), col.allgather(16, 2)), col.allgather(16, 2))),
          "i32", "u32", 4 * 7 + 3, options={"slice_vectors": slice_vectors})


def test_copies_that_cannot_be_propagated_and_permuted_positions():
    from test_host_plan import awkward_copy_schedules
    for topo, coll, sched in awkward_copy_schedules():
        for dtype, dist in (("f32", "uniform"), ("f16", "normal"), ("i32", "u32")):
            check(topo, coll, sched, dtype, dist, 4 * 5 + 2)
    topo, ag = tp.hcm8(), col.allgather(8, 2)
    sched, coll = gen.compose_allreduce(gen.greedy_bfs(topo, ag), ag)
    G = coll.num_chunks
    rng = np.random.default_rng(5)
    slot = np.stack([rng.permutation(G + 3)[:G] for _ in range(8)], axis=1).astype(np.int32)
    check(topo, coll, sched, "f16", "normal", 8 * 6 + 2, slot=slot, slots_per_rank=G + 3)


@pytest.mark.parametrize("seed", range(100, 140))
def test_random_schedules_through_both_tables(seed):
    label, topo, coll, sched, dtype, dist, epc = random_case(seed)
    check(topo, coll, sched, dtype, dist, min(epc, 4 * 13 + 1), seed=seed)


def test_table_accessor_arguments():
    topo, ag = tp.ring(4), col.allgather(4, 1)
    plan = sccl.sccl_plan_create(*to_binding(topo, ag, gen.greedy_bfs(topo, ag), "f32", 16), options={"flags": HOST})
    with pytest.raises(sccl.ScclError):
        sccl.sccl_plan_table(plan, 7)
    words, info = sccl.sccl_plan_table(plan, sccl.SCCL_LOWER_MEMORY)
    # four chunks; each goes to both neighbours in step 0 (header, source, two destinations) and on to the far node in
    # step 1 (header, source, one destination): seven words per chunk, after five offsets padded to eight words
    assert info[0] == 8 and [int(x) for x in words[:5]] == [0, 7, 14, 21, 28] and len(words) == 8 + 28
    first = [int(x) for x in words[8:12]]
    assert first[0] == (2 << 8) and first[1] == (0 | 0 << 8) and sorted(w & 0xff for w in first[2:]) == [1, 3]
    sccl.sccl_plan_destroy(plan)


def test_wide_range_inputs_make_a_planted_table_mistake_visible():
    """Inputs whose neighbours differ by many binades: nearly every sum rounds, so the order of additions shows in the
    bits.  The tables pass; a copy of the staged table with one task's first two sources swapped, a source dropped, or
    one store taken from another storage, does not (the mistake is planted in the copy that is interpreted here, on the CPU)."""
    topo, ag = tp.torus2d(4, 4), col.allgather(16, 4)
    ar, arc = gen.compose_allreduce(gen.greedy_bfs(topo, ag), ag)
    G = arc.num_chunks
    for dtype, epc in (("f32", 4 * 9 + 1), ("f16", 8 * 40 + 2)):
        check(topo, arc, ar, dtype, "wide", epc)
        bufs = [inputs.generate("wide", dtype, 5, n, 0, G * epc) for n in range(16)]
        want = [b.copy() for b in bufs]
        ex.execute(dtype, G, epc, ar, want)
        plan = sccl.sccl_plan_create(*to_binding(topo, arc, ar, dtype, epc), options={"flags": HOST})
        st = sccl.sccl_plan_stats(plan)
        words, info = sccl.sccl_plan_table(plan, sccl.SCCL_LOWER_STAGED)
        sccl.sccl_plan_destroy(plan)
        u = np.uint32 if dtype == "f32" else np.uint16

        def differs(table):
            got = [b.copy() for b in bufs]
            interpret_staged_table(table, info, G, dtype, epc, got, st["vector_bytes"])
            return any((g.view(u) != w.view(u)).any() for g, w in zip(got, want))

        assert not differs(words)
        b = words[:info[0]]
        out = 8 + info[1] + int(b[3]) + 2
        task = (out + 2 * int(b[2]) + 3) & ~3
        swapped = [t for t in range(int(b[4])) if (int(b[task + 8 * t]) >> 24) >= 2]
        assert swapped
        seen = 0
        for t in swapped:
            bad = words.copy()
            bad[task + 8 * t + 2], bad[task + 8 * t + 3] = words[task + 8 * t + 3], words[task + 8 * t + 2]
            seen += differs(bad)
        # binary16 operands are summed in binary32 and narrowed once: the order inside one group then moves the binary32
        # sum by far less than a binary16 ulp, so only binary32 data can show a swap (a wrong SOURCE shows in both)
        assert seen == (len(swapped) if dtype == "f32" else 0)
        for t in swapped:
            bad = words.copy()
            bad[task + 8 * t + 2] = info[3]                                       # the identity storage instead of the first source
            assert differs(bad)
        bad = words.copy()
        bad[out] = 0 if int(words[out]) != 0 else (1 << info[2]) * st["vector_bytes"]      # first store from another storage
        assert differs(bad)
