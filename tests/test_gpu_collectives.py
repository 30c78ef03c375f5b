"""GPU parity for the other collectives of Table 2 and Reduce: same library, same kernel, other (pre, post)."""
import numpy as np
import pytest

from gpu_util import assert_same_bits, bits, run_both
from oracle import collective as col
from oracle import generate as gen
from oracle import topology as tp
from oracle.validate import validate
from paper_2008_08708_amd import inputs

pytestmark = pytest.mark.gpu

TOPOS = [tp.ring(8), tp.hcm8(), tp.dgx1(), tp.torus2d(4, 4)]


def poisoned(coll, dtype, dist, seed, epc):
    P, G = coll.num_nodes, coll.num_chunks
    bufs = [inputs.generate(dist, dtype, seed, n, 0, G * epc) for n in range(P)]
    for n in range(P):
        for c in range(G):
            if not coll.pre[c, n]:
                inputs.poison(bufs[n], c * epc, (c + 1) * epc)
    return bufs


@pytest.mark.parametrize("topo", TOPOS, ids=[t.name for t in TOPOS])
@pytest.mark.parametrize("which", ["broadcast", "gather", "scatter", "alltoall"])
def test_non_combining_collectives(topo, which):
    P = topo.num_nodes
    coll = {"broadcast": lambda: col.broadcast(P, 3, 1), "gather": lambda: col.gather(P, 2, P - 1),
            "scatter": lambda: col.scatter(P, 2 * P, 0), "alltoall": lambda: col.alltoall(P, P)}[which]()
    s = gen.greedy_route(topo, coll)
    assert validate(topo, coll, s).ok
    epc = 2048 + 4 * 21
    bufs = poisoned(coll, "f32", "uniform", 41, epc)
    want, got = run_both(topo, coll, s, "f32", bufs, epc, label=f"{which}-{topo.name}")
    assert_same_bits(want, got)
    for c in range(coll.num_chunks):                      # closed form on the post-condition
        owner = int(np.nonzero(coll.pre[c])[0][0])
        for m in range(P):
            if coll.post[c, m]:
                assert (bits(got[m][c * epc:(c + 1) * epc]) == bits(bufs[owner][c * epc:(c + 1) * epc])).all()


@pytest.mark.parametrize("topo", TOPOS, ids=[t.name for t in TOPOS])
@pytest.mark.parametrize("dtype,dist", [("f32", "uniform"), ("f16", "normal"), ("i32", "u32")])
def test_reduce_to_a_root(topo, dtype, dist):
    P, C, root = topo.num_nodes, 3, 2
    bc = col.broadcast(P, C, root)
    red = gen.invert(gen.greedy_route(topo, bc), bc)
    rc = col.reduce(P, C, root)
    rtopo = topo.reversed()
    assert validate(rtopo, rc, red).ok
    epc = 1024 + 8 * 3
    bufs = [inputs.generate(dist, dtype, 43, n, 0, C * epc) for n in range(P)]
    want, got = run_both(rtopo, rc, red, dtype, bufs, epc, label=f"reduce-{topo.name}")
    assert_same_bits(want, got)
    if dtype == "i32":
        direct = np.zeros(C * epc, dtype=np.uint32)
        for b in bufs:
            direct = direct + b.view(np.uint32)
        assert (got[root].view(np.uint32) == direct).all()


@pytest.mark.parametrize("topo", TOPOS, ids=[t.name for t in TOPOS])
def test_alltoall_in_a_compact_layout(topo):
    P = topo.num_nodes
    coll = col.alltoall(P, P)
    s = gen.greedy_route(topo, coll)
    slot, per_rank = col.compact_slots(coll, s.sends)
    epc = 1024 + 4 * 9
    rng_bufs = [inputs.generate("uniform", "f32", 47, n, 0, per_rank * epc) for n in range(P)]
    for n in range(P):                                    # positions of chunks the rank does not hold at the start are undefined
        owned = {int(slot[c, n]) for c in range(coll.num_chunks) if coll.pre[c, n]}
        for k in range(per_rank):
            if k not in owned:
                inputs.poison(rng_bufs[n], k * epc, (k + 1) * epc)
    want, got = run_both(topo, coll, s, "f32", rng_bufs, epc, label=f"alltoall-compact-{topo.name}", slot=slot, slots_per_rank=per_rank)
    assert_same_bits(want, got)
    for j in range(P):                                    # rank j's block n came from rank n
        for n in range(P):
            c = j * P + n
            a = got[j][slot[c, j] * epc:(slot[c, j] + 1) * epc]
            b = rng_bufs[n][slot[c, n] * epc:(slot[c, n] + 1) * epc]
            assert (bits(a) == bits(b)).all()


@pytest.mark.parametrize("mode", ["sccl_execute", "sccl_execute_stepwise"])
def test_allreduce_with_permuted_positions(mode):
    # every rank keeps the chunks in its own random order: nothing may assume position == chunk id
    topo = tp.hcm8()
    ag = col.allgather(8, 2)
    sched, coll = gen.compose_allreduce(gen.greedy_bfs(topo, ag), ag)
    G, P, epc = coll.num_chunks, 8, 2048 + 12
    rng = np.random.default_rng(5)
    slot = np.stack([rng.permutation(G + 3)[:G] for _ in range(P)], axis=1).astype(np.int32)
    bufs = [inputs.generate("normal", "f16", 49, n, 0, (G + 3) * epc) for n in range(P)]
    want, got = run_both(topo, coll, sched, "f16", bufs, epc, label="allreduce-permuted", mode=mode, slot=slot, slots_per_rank=G + 3)
    assert_same_bits(want, got)
    ref = got[0][slot[0, 0] * epc:(slot[0, 0] + 1) * epc]
    for n in range(1, P):
        assert (bits(got[n][slot[0, n] * epc:(slot[0, n] + 1) * epc]) == bits(ref)).all()


def test_memcpy_lowering_with_a_compact_layout():
    topo = tp.ring(8)
    coll = col.alltoall(8, 8)
    s = gen.greedy_route(topo, coll)
    slot, per_rank = col.compact_slots(coll, s.sends)
    epc = 512 + 4
    bufs = [inputs.generate("u32", "i32", 55, n, 0, per_rank * epc) for n in range(8)]
    want, got = run_both(topo, coll, s, "i32", bufs, epc, label="alltoall-compact-memcpy", mode="sccl_execute_memcpy", slot=slot, slots_per_rank=per_rank)
    assert_same_bits(want, got)


@pytest.mark.parametrize("epc", [2, 64, 1000])
def test_small_chunks_of_other_collectives(epc):
    topo = tp.hcm8()
    for coll in (col.broadcast(8, 3, 1), col.alltoall(8, 8), col.gather(8, 2, 7)):
        s = gen.greedy_route(topo, coll)
        bufs = poisoned(coll, "f16", "normal", 73, epc)
        want, got = run_both(topo, coll, s, "f16", bufs, epc, label=f"small-{coll.name}-{epc}")
        assert_same_bits(want, got)
        slot, per_rank = col.compact_slots(coll, s.sends)
        cb = [inputs.generate("normal", "f16", 75, n, 0, per_rank * epc) for n in range(8)]
        want, got = run_both(topo, coll, s, "f16", cb, epc, label=f"small-compact-{coll.name}-{epc}", slot=slot, slots_per_rank=per_rank)
        assert_same_bits(want, got)


# ---- topologies that are not symmetric, and bandwidth constraints over SETS of links, through the library

def _directed_ring(P):
    return tp.point_to_point(P, {(n, (n + 1) % P): 1 for n in range(P)}, f"dring{P}")


def _dgx1_one_way_outer_cycle():
    """The DGX-1 graph with the single-link Hamiltonian cycle 0,2,1,3,6,4,7,5 (section 2.2) kept in ONE direction only:
    every node keeps all its double links, but the graph is no longer symmetric."""
    cyc = [0, 2, 1, 3, 6, 4, 7, 5]
    dropped = {(cyc[(i + 1) % 8], cyc[i]) for i in range(8)}
    full = tp.dgx1()
    bw = tuple((L, b) for (L, b) in full.bw if not (len(L) == 1 and next(iter(L)) in dropped and b == 1))
    assert len(bw) == len(full.bw) - 8
    return tp.Topology(8, bw, "dgx1-oneway")


def _status(topo, coll, sched, dtype, epc):
    from helpers import plan_status
    return plan_status(topo, coll, sched, dtype, epc)[0]


@pytest.mark.parametrize("make", [lambda: _directed_ring(6), _dgx1_one_way_outer_cycle], ids=["directed-ring6", "dgx1-one-way-cycle"])
@pytest.mark.parametrize("dtype,dist", [("f32", "uniform"), ("f16", "normal"), ("i32", "u32")])
def test_reduce_needs_the_reversed_topology(make, dtype, dist):
    # section 3.5: a Reduce is a Broadcast inverted, on the topology with every link turned round.  On a graph
    # that is not symmetric the inverted schedule is valid ONLY there: the library must say so on both graphs.
    topo = make()
    assert not topo.is_symmetric()
    P, C, root = topo.num_nodes, 2, 1
    bc = col.broadcast(P, C, root)
    fwd = gen.greedy_route(topo, bc)
    assert validate(topo, bc, fwd).ok
    red, rc = gen.invert(fwd, bc), col.reduce(P, C, root)
    rtopo = topo.reversed()
    assert validate(rtopo, rc, red).ok and not validate(topo, rc, red).ok
    epc = 2048 + 4 * 5
    assert _status(rtopo, rc, red, dtype, epc) == "SCCL_OK"
    assert _status(topo, rc, red, dtype, epc) == "SCCL_ERR_SEND_NO_LINK"
    bufs = [inputs.generate(dist, dtype, 57, n, 0, C * epc) for n in range(P)]
    want, got = run_both(rtopo, rc, red, dtype, bufs, epc, label=f"reduce-{topo.name}")
    assert_same_bits(want, got)
    if dtype == "i32":                                     # order-free: the root holds the plain sum
        direct = np.zeros(C * epc, dtype=np.uint32)
        for b in bufs:
            direct = direct + b.view(np.uint32)
        assert (got[root].view(np.uint32) == direct).all()
    # the forward Broadcast runs on the graph as it is (and not on the reversed one)
    assert _status(rtopo, bc, fwd, dtype, epc) == "SCCL_ERR_SEND_NO_LINK"
    bb = poisoned(bc, dtype, dist, 59, epc)
    want, got = run_both(topo, bc, fwd, dtype, bb, epc, label=f"broadcast-{topo.name}")
    assert_same_bits(want, got)


def _two_islands():
    """The model of section 5.2.2: two fully connected islands {0,2,3} and {4,6,7}; node 1 (5) reaches its island
    over ONE shared bus (one chunk per round for all six directed links together), and 1 <-> 5 is a bridge."""
    links = {}
    for isl in ((0, 2, 3), (4, 6, 7)):
        for a in isl:
            for b in isl:
                if a != b:
                    links[(a, b)] = 1
    bw = [(frozenset([e]), b) for e, b in sorted(links.items())]
    left = frozenset([(0, 1), (1, 0), (1, 2), (2, 1), (1, 3), (3, 1)])
    right = frozenset([(4, 5), (5, 4), (5, 6), (6, 5), (5, 7), (7, 5)])
    return tp.Topology(8, tuple(bw) + ((left, 1), (right, 1), (frozenset([(1, 5)]), 1), (frozenset([(5, 1)]), 1)), "two-islands")


@pytest.mark.parametrize("which", ["bus4-one-step", "bus4-greedy", "two-islands"])
def test_set_valued_bandwidth_constraints(which):
    # section 3.2.1: a constraint may cover a SET of links (a shared bus).  Allgather and the Allreduce composed from
    # it, validated by both sides and executed on the GPU; one round fewer must be refused with SCCL_ERR_BANDWIDTH.
    from oracle import synthesize as syn
    from oracle.schedule import Schedule
    if which == "two-islands":
        topo = _two_islands()
        ag = col.allgather(8, 1)
        s = gen.greedy_bfs(topo, ag)
    else:
        topo = tp.shared_bus(4)
        ag = col.allgather(4, 1)
        s = syn.solve_instance(topo, ag, 1, 12) if which == "bus4-one-step" else gen.greedy_bfs(topo, ag, rounds=[3] * 8)
    assert validate(topo, ag, s).ok
    epc = 1024 + 4 * 11
    assert _status(topo, ag, s, "f32", epc) == "SCCL_OK"
    busiest = int(np.argmax(np.bincount(s.sends[:, 3], minlength=s.num_steps) / np.array(s.rounds)))
    tight = list(s.rounds)
    if which != "two-islands":                            # on the bus every send of a step shares one budget
        tight[busiest] = int(np.bincount(s.sends[:, 3], minlength=s.num_steps)[busiest]) - 1
        if tight[busiest] >= 1:
            short = Schedule(tight, s.sends)
            assert not validate(topo, ag, short).ok
            assert _status(topo, ag, short, "f32", epc) == "SCCL_ERR_BANDWIDTH"
    bufs = poisoned(ag, "f32", "uniform", 61, epc)
    want, got = run_both(topo, ag, s, "f32", bufs, epc, label=f"allgather-{which}")
    assert_same_bits(want, got)
    ar, arc = gen.compose_allreduce(s, ag)
    assert validate(topo, arc, ar).ok and _status(topo, arc, ar, "f16", epc) == "SCCL_OK"
    rb = [inputs.generate("normal", "f16", 63, n, 0, arc.num_chunks * epc) for n in range(topo.num_nodes)]
    want, got = run_both(topo, arc, ar, "f16", rb, epc, label=f"allreduce-{which}")
    assert_same_bits(want, got)
    for g in got[1:]:
        assert (bits(g) == bits(got[0])).all()


def test_the_papers_table_rows_execute():
    # every stored witness of Tables 4 and 5 (and the Allreduce composed from every Allgather witness) through the
    # library on the GPU, under both lowerings, against the oracle
    import glob
    import os
    from oracle import reproduce_tables as rt
    topos = {"ring8": tp.ring(8), "dgx1": tp.dgx1()}
    paths = sorted(glob.glob(os.path.join(rt.WITNESSES, "*.txt")))
    assert len(paths) >= 36
    for path in paths:
        tname, name, C, S, R = os.path.basename(path)[:-4].split("_")
        topo, coll = topos[tname], rt.MAKE[name](8, int(C))
        sched = rt.read_witness(path)
        epc = 4 * 19 + 4
        bufs = poisoned(coll, "f32", "uniform", 71, epc)
        want, got = run_both(topo, coll, sched, "f32", bufs, epc, label=os.path.basename(path))
        assert_same_bits(want, got)
        if name == "allgather":
            ar, arc = gen.compose_allreduce(sched, coll)
            rb = [inputs.generate("uniform", "f32", 73, n, 0, arc.num_chunks * epc) for n in range(8)]
            want, got = run_both(topo, arc, ar, "f32", rb, epc, label="allreduce-of-" + os.path.basename(path))
            assert_same_bits(want, got)
