"""Pins for oracle/synthesize.py: the exact search must find the rows the paper's tables list as feasible,
prove the neighbouring instances they imply to be infeasible, and Algorithm 1 must report the tables' frontier."""
from fractions import Fraction

import pytest

from conftest import read_table
from oracle import collective as col
from oracle import generate as gen
from oracle import synthesize as syn
from oracle import topology as tp
from oracle.validate import validate

T4 = {(r[0], r[1], r[2], r[3]): r[6] for r in read_table("table4_dgx1.txt")}
T5 = {(r[0], r[1], r[2], r[3]): r[6] for r in read_table("table5_z52.txt")}

MAKE = {
    "allgather": lambda P, C: col.allgather(P, C),
    "broadcast": lambda P, C: col.broadcast(P, C, 0),
    "gather": lambda P, C: col.gather(P, C, 0),
    "alltoall": lambda P, C: col.alltoall(P, C),
}

# rows small enough for the CPU suite (each solves in seconds)
FEASIBLE = [
    (tp.dgx1(), T4, "allgather", 1, 2, 2), (tp.dgx1(), T4, "allgather", 2, 3, 3), (tp.dgx1(), T4, "allgather", 2, 2, 3),
    (tp.dgx1(), T4, "broadcast", 2, 2, 2), (tp.dgx1(), T4, "broadcast", 6, 3, 3), (tp.dgx1(), T4, "broadcast", 6, 3, 5),
    (tp.dgx1(), T4, "gather", 1, 2, 2), (tp.dgx1(), T4, "gather", 2, 2, 3), (tp.dgx1(), T4, "gather", 6, 3, 7),
    (tp.dgx1(), T4, "alltoall", 8, 3, 3), (tp.dgx1(), T4, "alltoall", 8, 2, 3),
    (tp.ring(8), T5, "allgather", 1, 4, 4), (tp.ring(8), T5, "allgather", 2, 7, 7), (tp.ring(8), T5, "allgather", 2, 4, 7),
    (tp.ring(8), T5, "broadcast", 2, 4, 4), (tp.ring(8), T5, "broadcast", 4, 5, 5), (tp.ring(8), T5, "broadcast", 6, 6, 6),
    (tp.ring(8), T5, "gather", 1, 4, 4), (tp.ring(8), T5, "gather", 2, 4, 7), (tp.ring(8), T5, "alltoall", 8, 4, 8),
]


@pytest.mark.parametrize("topo,table,name,C,S,R", FEASIBLE, ids=[f"{t.name}-{n}-{C}-{S}-{R}" for t, _, n, C, S, R in FEASIBLE])
def test_rows_of_the_tables_are_feasible(topo, table, name, C, S, R):
    assert (name, C, S, R) in table                       # it really is a row the paper prints
    coll = MAKE[name](topo.num_nodes, C)
    s = syn.solve_instance(topo, coll, S, R)
    assert s is not None
    rep = validate(topo, coll, s)
    assert rep.ok, rep.detail
    assert (s.num_steps, s.num_rounds) == (S, R)


INFEASIBLE = [
    # "latency optimal" rows: one step fewer does not exist
    (tp.dgx1(), "allgather", 1, 1, 1), (tp.dgx1(), "allgather", 1, 1, 6), (tp.dgx1(), "broadcast", 2, 1, 4),
    (tp.dgx1(), "alltoall", 8, 1, 8), (tp.ring(8), "allgather", 1, 3, 3), (tp.ring(8), "allgather", 1, 3, 12),
    (tp.ring(8), "alltoall", 8, 3, 12),
    # "bandwidth optimal" rows: one round fewer does not exist
    (tp.dgx1(), "allgather", 6, 3, 6), (tp.dgx1(), "allgather", 2, 2, 2), (tp.ring(8), "allgather", 2, 4, 6),
    (tp.ring(8), "allgather", 2, 7, 6), (tp.ring(8), "gather", 2, 4, 6),
    # Broadcast of 3 chunks in 2 steps and 2 rounds: the table's 2-step row carries 2 chunks
    (tp.dgx1(), "broadcast", 3, 2, 2),
    # Alltoall (8,2,3) is latency optimal and needs its third round
    (tp.dgx1(), "alltoall", 8, 2, 2),
]


@pytest.mark.parametrize("topo,name,C,S,R", INFEASIBLE, ids=[f"{t.name}-{n}-{C}-{S}-{R}" for t, n, C, S, R in INFEASIBLE])
def test_instances_the_tables_rule_out_are_infeasible(topo, name, C, S, R):
    assert syn.solve_instance(topo, MAKE[name](topo.num_nodes, C), S, R) is None


def test_exact_search_agrees_with_breadth_first_search_on_tiny_rings():
    from oracle import search
    for P in (3, 4, 5):
        topo, ag = tp.ring(P), col.allgather(P, 1)
        smin, _ = search.min_steps(topo, ag)
        assert syn.solve_instance(topo, ag, smin, smin) is not None
        if smin > 1:
            assert syn.solve_instance(topo, ag, smin - 1, smin - 1) is None
    # the worked example of section 3.1: two steps need three rounds for 2 chunks per link... one chunk per node fits (1,2,2)
    assert syn.solve_instance(tp.ring(4), col.allgather(4, 1), 2, 2) is not None


def test_algorithm_1_on_the_eight_ring():
    topo = tp.ring(8)
    make = lambda C: col.allgather(8, C)
    # k = 0: starts at the latency-optimal (1,4,4) and ends at the bandwidth-optimal (2,7,7)
    found = [(C, S, R) for (C, S, R, s) in syn.pareto_synthesize(0, topo, make)]
    assert found[0] == (1, 4, 4) and found[-1] == (2, 7, 7)
    assert T5[("allgather", 1, 4, 4)] == "latency" and T5[("allgather", 2, 7, 7)] == "bandwidth"
    # every reported algorithm is at least as good in bandwidth as the one before (the frontier walks down)
    ratios = [Fraction(R, C) for (C, S, R) in found]
    assert ratios == sorted(ratios, reverse=True)
    # k = 3: the first step count already reaches the bandwidth bound: (2,4,7), "both"
    found = syn.pareto_synthesize(3, topo, make)
    assert [(C, S, R) for (C, S, R, s) in found] == [(2, 4, 7)] and T5[("allgather", 2, 4, 7)] == "both"
    assert validate(topo, make(2), found[0][3]).ok


def test_algorithm_1_on_the_dgx1_graph_first_rows():
    topo = tp.dgx1()
    make = lambda C: col.allgather(8, C)
    found = [(C, S, R) for (C, S, R, s) in syn.pareto_synthesize(0, topo, make, max_steps=3)]
    assert found == [(1, 2, 2), (2, 3, 3)]                 # the first two rows of Table 4
    found = [(C, S, R) for (C, S, R, s) in syn.pareto_synthesize(1, topo, make, max_steps=2)]
    assert found == [(2, 2, 3)]                            # Table 4's second latency-optimal row


def test_synthesized_schedules_compose_into_the_allreduce_rows():
    # (2,2,3) on the DGX-1 graph gives Allreduce (16,4,6); (2,4,7) on the 8-ring gives (16,8,14)
    for topo, table, (C, S, R) in ((tp.dgx1(), T4, (2, 2, 3)), (tp.ring(8), T5, (2, 4, 7))):
        ag = col.allgather(8, C)
        s = syn.solve_instance(topo, ag, S, R)
        ar, arc = gen.compose_allreduce(s, ag)
        assert validate(topo, arc, ar).ok
        assert ("allreduce",) + ar.csr(arc.num_chunks) in table
        assert max(ar.rounds) > 1                          # a k > 0 schedule: some step has several rounds


def test_shared_constraints_are_respected_by_search_and_generators():
    # section 3.2.1's shared bus: all pairs may talk, one chunk per round in total.  An Allgather of 4 nodes
    # moves 12 chunks, one per round: 12 rounds are enough in a single step, 11 are not.
    bus, ag = tp.shared_bus(4), col.allgather(4, 1)
    s = syn.solve_instance(bus, ag, 1, 12)
    assert s is not None and validate(bus, ag, s).ok and s.rounds == [12]
    assert syn.solve_instance(bus, ag, 1, 11) is None
    assert syn.solve_instance(bus, ag, 3, 11) is None
    # the greedy generators spend the shared budget once per send, whatever the link
    g = gen.greedy_bfs(bus, ag, rounds=[3] * 8)
    assert validate(bus, ag, g).ok and g.num_rounds >= 12
    # the model of section 5.2.2: two fully connected islands whose bridge nodes share one bus per side
    links = {}
    for isl in ((0, 2, 3), (4, 6, 7)):
        for a in isl:
            for b in isl:
                if a != b:
                    links[(a, b)] = 1
    bw = [(frozenset([e]), b) for e, b in links.items()]
    left = frozenset([(0, 1), (1, 0), (1, 2), (2, 1), (1, 3), (3, 1)])          # the paper's left-socket entry
    right = frozenset([(4, 5), (5, 4), (5, 6), (6, 5), (5, 7), (7, 5)])
    bridge = frozenset([(1, 5)]), frozenset([(5, 1)])
    topo = tp.Topology(8, tuple(bw) + ((left, 1), (right, 1), (bridge[0], 1), (bridge[1], 1)), "z52-pcie")
    ag8 = col.allgather(8, 1)
    g = gen.greedy_bfs(topo, ag8)
    rep = validate(topo, ag8, g)
    assert rep.ok, rep.detail
    # everything the right half learns about the left half crosses 1 -> 5, one chunk per round: at least 4 rounds
    assert g.num_rounds >= 4 and g.num_steps >= tp.diameter(topo)
    exact = syn.solve_instance(topo, ag8, g.num_steps, g.num_rounds)
    assert exact is not None and validate(topo, ag8, exact).ok
