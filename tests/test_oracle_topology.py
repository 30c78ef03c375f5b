"""Pins for oracle/topology.py and oracle/collective.py: facts the paper states about its graphs and relations."""
from fractions import Fraction

import numpy as np
import pytest

from conftest import read_examples
from oracle import collective as col
from oracle import topology as tp


def test_ring_degrees_and_link_count():
    for P in (3, 4, 8):
        t = tp.ring(P)
        assert len(t.edges()) == 2 * P
        for n in range(P):
            assert t.in_neighbours(n) == sorted({(n - 1) % P, (n + 1) % P})


def test_dgx1_facts_from_the_paper():
    ex = read_examples()
    t = tp.dgx1()
    links = dict((next(iter(L)), b) for L, b in t.bw)
    # both groups are fully connected
    for base in (0, 4):
        for i in range(4):
            for j in range(4):
                if i != j:
                    assert (base + i, base + j) in links
    # four inter-group links (undirected)
    cross = {frozenset(e) for e in links if (e[0] < 4) != (e[1] < 4)}
    assert len(cross) == int(ex["dgx1_cross_links"][0])
    # six link units into and out of every node
    for n in range(8):
        assert sum(b for (s, d), b in links.items() if d == n) == int(ex["dgx1_link_units_per_node"][0])
        assert sum(b for (s, d), b in links.items() if s == n) == int(ex["dgx1_link_units_per_node"][0])
        assert tp.ingress_per_round(t, n) == 6
    assert tp.diameter(t) == int(ex["dgx1_diameter"][0])
    assert tp.allgather_bandwidth_bound(t) == Fraction(ex["dgx1_allgather_bw_bound"][0])
    assert t.is_symmetric()


def test_hcm8_matches_the_configuration_text():
    t = tp.hcm8()
    links = dict((next(iter(L)), b) for L, b in t.bw)
    assert len(links) == 32
    for n in range(8):
        assert len(t.in_neighbours(n)) == 4          # 3 in the clique + 1 cross
        assert tp.ingress_per_round(t, n) == 6
    for e in ((0, 3), (1, 2), (4, 7), (5, 6), (0, 4), (1, 5), (2, 6), (3, 7)):
        assert links[e] == 2 and links[(e[1], e[0])] == 2
    assert sum(1 for b in links.values() if b == 1) == 16
    assert tp.diameter(t) == 2
    assert tp.allgather_bandwidth_bound(t) == Fraction(7, 6)
    assert t.is_symmetric()


@pytest.mark.parametrize("topo,diam,bound", [
    (tp.ring(4), 2, Fraction(3, 2)),
    (tp.ring(8), 4, Fraction(7, 2)),
    (tp.ring(6), 3, Fraction(5, 2)),
    (tp.torus2d(4, 4), 4, Fraction(15, 4)),
    (tp.complete(8), 1, Fraction(1, 1)),
])
def test_diameter_and_ingress_bound(topo, diam, bound):
    assert tp.diameter(topo) == diam
    assert tp.allgather_bandwidth_bound(topo) == bound


def test_torus_numbering():
    t = tp.torus2d(4, 4)
    assert len(t.edges()) == 64
    assert t.in_neighbours(0) == [1, 3, 4, 12]
    assert t.in_neighbours(5) == [1, 4, 6, 9]


def test_shared_bus_and_zero_bandwidth_links():
    bus = tp.shared_bus(4)
    assert tp.ingress_per_round(bus, 0) == 1
    # a link mentioned by a zero-bandwidth constraint is not usable (definition of E)
    t = tp.Topology(3, ((frozenset([(0, 1)]), 1), (frozenset([(1, 2)]), 1), (frozenset([(1, 2), (2, 0)]), 0)))
    assert t.edges() == [(0, 1)]
    with pytest.raises(ValueError):
        tp.diameter(t)


def test_reversed_topology():
    t = tp.point_to_point(3, {(0, 1): 1, (1, 2): 2})
    r = t.reversed()
    assert r.edges() == [(1, 0), (2, 1)]
    assert not t.is_symmetric()


def test_relations_table1():
    G, P = 8, 4
    sc = col.rel_scattered(G, P)
    tr = col.rel_transpose(G, P)
    for c in range(G):
        for n in range(P):
            assert sc[c, n] == (n == c % P)
            assert tr[c, n] == (n == (c // P) % P)
    assert col.rel_all(G, P).sum() == G * P
    assert (col.rel_root(G, P, 2)[:, 2] == 1).all() and col.rel_root(G, P, 2).sum() == G
    # every chunk has exactly one owner under Scattered and Transpose
    assert (sc.sum(axis=1) == 1).all() and (tr.sum(axis=1) == 1).all()


def test_collectives_table2_and_chunk_numbering():
    P, C = 4, 3
    ag = col.allgather(P, C)
    assert ag.num_chunks == P * C                    # Allgather: G = P*C
    # node n's i-th chunk is i*P + n
    for n in range(P):
        owned = [c for c in range(ag.num_chunks) if ag.pre[c, n]]
        assert owned == [i * P + n for i in range(C)]
    assert ag.post.all()
    bc = col.broadcast(P, C, root=1)
    assert bc.num_chunks == C                        # Broadcast: G = C
    assert (bc.pre == col.rel_root(C, P, 1)).all() and bc.post.all()
    a2a = col.alltoall(P, P)
    assert (a2a.pre == col.rel_scattered(P * P, P)).all() and (a2a.post == col.rel_transpose(P * P, P)).all()
    g = col.gather(P, 1, root=3)
    assert (g.post == col.rel_root(P, P, 3)).all()
    sc = col.scatter(P, 2, root=0)
    assert (sc.pre == col.rel_root(2, P, 0)).all() and (sc.post == col.rel_scattered(2, P)).all()
    ar = col.allreduce(P, 8)
    assert ar.combining and ar.pre.all() and ar.post.all()
    rs = col.reducescatter(P, 8)
    assert rs.combining and rs.pre.all() and (rs.post == col.rel_scattered(8, P)).all()
