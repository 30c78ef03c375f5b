"""Pins for the remaining collectives of Table 2 (Gather, Scatter, Broadcast, Alltoall) and Reduce (section 3.5):
closed forms of the results, lower bounds, and the feasible rows the paper's tables list."""
from fractions import Fraction

import numpy as np
import pytest

from conftest import read_table
from oracle import collective as col
from oracle import executor as ex
from oracle import generate as gen
from oracle import topology as tp
from oracle.schedule import REDUCE
from oracle.validate import validate
from paper_2008_08708_amd import inputs

T4 = read_table("table4_dgx1.txt")
T5 = read_table("table5_z52.txt")
TOPOS = [tp.ring(4), tp.ring(8), tp.hcm8(), tp.dgx1(), tp.torus2d(4, 4), tp.complete(6)]


def poisoned_inputs(coll, dtype, dist, seed, epc):
    P, G = coll.num_nodes, coll.num_chunks
    bufs = [inputs.generate(dist, dtype, seed, n, 0, G * epc) for n in range(P)]
    for n in range(P):
        for c in range(G):
            if not coll.pre[c, n]:
                inputs.poison(bufs[n], c * epc, (c + 1) * epc)
    return bufs


def chunk(b, c, epc):
    v = b[c * epc:(c + 1) * epc]
    return v.view(np.uint32 if v.dtype.itemsize == 4 else np.uint16)


@pytest.mark.parametrize("topo", TOPOS, ids=[t.name for t in TOPOS])
def test_broadcast_gather_scatter_alltoall_closed_forms(topo):
    P, epc = topo.num_nodes, 9
    dist = tp.distances(topo)
    for coll in (col.broadcast(P, 3, root=1), col.gather(P, 2, root=P - 1), col.scatter(P, 2 * P, root=0), col.alltoall(P, P)):
        s = gen.greedy_route(topo, coll)
        rep = validate(topo, coll, s)
        assert rep.ok, (coll.name, rep.detail)
        # every receive happens once, and only at nodes that need or relay the chunk
        recv = [(c, m) for (c, n, m, st, op) in s.sends.tolist()]
        assert len(recv) == len(set(recv))
        # latency bound: the farthest (holder, target) pair
        far = max(dist[n][m] for c in range(coll.num_chunks) for n in range(P) for m in range(P)
                  if coll.pre[c, n] and coll.post[c, m])
        assert s.num_steps >= far
        bufs = poisoned_inputs(coll, "f32", "uniform", 13, epc)
        pristine = [b.copy() for b in bufs]
        ex.execute("f32", coll.num_chunks, epc, s, bufs)
        for c in range(coll.num_chunks):
            owner = int(np.nonzero(coll.pre[c])[0][0])
            for m in range(P):
                if coll.post[c, m]:
                    assert (chunk(bufs[m], c, epc) == chunk(pristine[owner], c, epc)).all(), (coll.name, c, m)
                    assert not inputs.is_poison(bufs[m][c * epc:(c + 1) * epc]).any()


def test_alltoall_is_a_transpose_of_blocks():
    # rank n's j-th send block is chunk j*P + n; after the Alltoall rank j holds it at the same chunk index,
    # i.e. rank j's block n came from rank n (the MPI meaning), read through Table 1's Scattered / Transpose
    P, epc = 4, 5
    topo, coll = tp.ring(4), col.alltoall(4, 4)
    s = gen.greedy_route(topo, coll)
    bufs = poisoned_inputs(coll, "i32", "u32", 3, epc)
    pristine = [b.copy() for b in bufs]
    ex.execute("i32", 16, epc, s, bufs)
    for j in range(P):
        for n in range(P):
            c = j * P + n
            assert (bufs[j][c * epc:(c + 1) * epc] == pristine[n][c * epc:(c + 1) * epc]).all()


@pytest.mark.parametrize("topo", [tp.ring(8), tp.hcm8(), tp.dgx1(), tp.torus2d(4, 4)], ids=lambda t: t.name)
@pytest.mark.parametrize("dtype,dist", [("i32", "u32"), ("f32", "smallint"), ("f16", "smallint")])
def test_reduce_is_the_inverse_of_broadcast_and_sums_at_the_root(topo, dtype, dist):
    P, C, root, epc = topo.num_nodes, 3, 2, 11
    bc = col.broadcast(P, C, root)
    s = gen.greedy_route(topo, bc)
    assert validate(topo, bc, s).ok
    red = gen.invert(s, bc)
    rc = col.reduce(P, C, root)
    assert validate(topo.reversed(), rc, red).ok
    assert (red.sends[:, 4] == REDUCE).all() and red.num_steps == s.num_steps
    bufs = [inputs.generate(dist, dtype, 7, n, 0, C * epc) for n in range(P)]
    if dtype == "i32":
        want = np.zeros(C * epc, dtype=np.uint32)
        for b in bufs:
            want = want + b.view(np.uint32)
    else:
        want = sum(b.astype(np.float64) for b in bufs)          # small integers: exact in any order
    ex.execute(dtype, C, epc, red, bufs)
    got = bufs[root].view(np.uint32) if dtype == "i32" else bufs[root].astype(np.float64)
    assert (got == want).all()


def test_latency_optimal_rows_of_the_tables_are_reached():
    rows4 = {(r[0], r[1], r[2], r[3]) for r in T4}
    rows5 = {(r[0], r[1], r[2], r[3]) for r in T5}
    # DGX-1: Broadcast (2,2,2) and Gather (1,2,2) are listed as latency optimal; the 8-ring machine: (2,4,4), (1,4,4)
    assert ("broadcast", 2, 2, 2) in rows4 and ("gather", 1, 2, 2) in rows4
    assert gen.greedy_route(tp.dgx1(), col.broadcast(8, 2, 0)).csr(2) == (2, 2, 2)
    assert gen.greedy_route(tp.dgx1(), col.gather(8, 1, 0)).csr(1) == (1, 2, 2)
    assert ("broadcast", 2, 4, 4) in rows5 and ("gather", 1, 4, 4) in rows5
    assert gen.greedy_route(tp.ring(8), col.broadcast(8, 2, 0)).csr(2) == (2, 4, 4)
    assert gen.greedy_route(tp.ring(8), col.gather(8, 1, 0)).csr(1) == (1, 4, 4)
    # no row of any collective undercuts the diameter
    for table, topo in ((T4, tp.dgx1()), (T5, tp.ring(8))):
        for (name, C, S, R, a, b, o) in table:
            assert S >= tp.diameter(topo) and R >= S


def test_gather_and_scatter_bandwidth_bound():
    # the root takes in (P-1)*C chunks over its in-links: R/C >= (P-1)/ingress (the rows marked bandwidth optimal)
    for table, topo in ((T4, tp.dgx1()), (T5, tp.ring(8))):
        bound = Fraction(topo.num_nodes - 1, tp.ingress_per_round(topo, 0))
        for (name, C, S, R, a, b, o) in table:
            if name == "gather":
                assert Fraction(R, C) >= bound
                if o in ("bandwidth", "both"):
                    assert Fraction(R, C) == bound
    for topo in (tp.dgx1(), tp.ring(8), tp.torus2d(4, 4)):
        P = topo.num_nodes
        s = gen.greedy_route(topo, col.gather(P, 1, 0))
        assert Fraction(s.num_rounds, 1) >= Fraction(P - 1, tp.ingress_per_round(topo, 0))


def test_greedy_route_agrees_with_greedy_bfs_on_allgather_validity():
    for topo in (tp.hcm8(), tp.ring(8)):
        ag = col.allgather(topo.num_nodes, 2)
        s = gen.greedy_route(topo, ag)
        assert validate(topo, ag, s).ok
        ar, arc = gen.compose_allreduce(s, ag)             # trees, so it can be inverted
        assert validate(topo, arc, ar).ok


def test_compact_layout_gives_the_same_chunks_in_other_places():
    for topo, coll in ((tp.ring(4), col.alltoall(4, 4)), (tp.hcm8(), col.alltoall(8, 8)), (tp.torus2d(4, 4), col.gather(16, 2, 3))):
        P, G, epc = coll.num_nodes, coll.num_chunks, 6
        s = gen.greedy_route(topo, coll)
        slot, per_rank = col.compact_slots(coll, s.sends)
        # every rank has room exactly for what it holds at some time; positions are distinct per rank
        for n in range(P):
            used = slot[:, n][slot[:, n] >= 0]
            assert len(set(used.tolist())) == used.size and used.size <= per_rank
        assert per_rank <= G
        if coll.name == "alltoall":
            assert per_rank < G                               # own chunks, received chunks, a few relayed ones
        full = poisoned_inputs(coll, "f32", "uniform", 19, epc)
        compact = []
        for n in range(P):
            b = np.empty(per_rank * epc, dtype=np.float32)
            inputs.poison(b, 0, b.size)
            for c in range(G):
                if coll.pre[c, n]:
                    b[slot[c, n] * epc:(slot[c, n] + 1) * epc] = full[n][c * epc:(c + 1) * epc]
            compact.append(b)
        ex.execute("f32", G, epc, s, full)
        ex.execute("f32", G, epc, s, compact, slot=slot, slots_per_rank=per_rank)
        for c in range(G):
            for n in range(P):
                if coll.post[c, n]:
                    a = chunk(full[n], c, epc)
                    b = chunk(compact[n], int(slot[c, n]), epc)
                    assert (a == b).all()
    # a send whose destination has no position is refused
    topo, coll = tp.ring(4), col.alltoall(4, 4)
    s = gen.greedy_route(topo, coll)
    slot, per_rank = col.compact_slots(coll, s.sends)
    slot[s.sends[0, 0], s.sends[0, 2]] = -1
    with pytest.raises(ValueError):
        ex.execute("f32", 16, 2, s, [np.zeros(per_rank * 2, np.float32) for _ in range(4)], slot=slot, slots_per_rank=per_rank)
