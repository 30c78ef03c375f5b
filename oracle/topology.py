"""Topologies as bandwidth relations (oracle side; test infrastructure).

Section 3.2.1 of the paper: a topology is a node count P and a bandwidth
relation B, a set of pairs (L, b) where L is a set of directed node pairs and
b bounds the number of chunks that may cross the edges of L in ONE round.  A
point-to-point link s->d of b chunks/round is ({(s, d)}, b).

Reading taken where the text is loose: the paper defines the usable edges E as
the pairs for which every constraint that mentions them has b > 0; a pair that
no constraint mentions would be vacuously usable with unbounded bandwidth, so
here a pair is a link only if at least one constraint mentions it (and all
that do have b > 0).
"""
from __future__ import annotations

from collections import deque
from dataclasses import dataclass, field
from fractions import Fraction
from typing import Dict, FrozenSet, List, Sequence, Tuple

Edge = Tuple[int, int]


@dataclass(frozen=True)
class Topology:
    """P nodes and the bandwidth relation B as a list of (edge set, chunks per round)."""

    num_nodes: int
    bw: Tuple[Tuple[FrozenSet[Edge], int], ...]
    name: str = ""

    def edges(self) -> List[Edge]:
        """Usable directed links E (section 3.4, definition of E)."""
        mentioned: Dict[Edge, bool] = {}
        for L, b in self.bw:
            for e in L:
                mentioned[e] = mentioned.get(e, True) and (b > 0)
        return sorted(e for e, ok in mentioned.items() if ok)

    def in_neighbours(self, n: int) -> List[int]:
        return sorted(s for (s, d) in self.edges() if d == n)

    def out_neighbours(self, n: int) -> List[int]:
        return sorted(d for (s, d) in self.edges() if s == n)

    def reversed(self) -> "Topology":
        """Every link turned round (section 3.5: Reduce inverts Broadcast on the reversed topology)."""
        return Topology(
            self.num_nodes,
            tuple((frozenset((d, s) for (s, d) in L), b) for L, b in self.bw),
            self.name + "^R",
        )

    def is_symmetric(self) -> bool:
        key = lambda t: sorted((sorted(L), b) for L, b in t.bw)
        return key(self) == key(self.reversed())


def point_to_point(num_nodes: int, links: Dict[Edge, int], name: str = "") -> Topology:
    """One singleton constraint ({(s,d)}, b) per directed link."""
    return Topology(num_nodes, tuple((frozenset([e]), b) for e, b in sorted(links.items())), name)


def ring(P: int, b: int = 1) -> Topology:
    """Bidirectional ring, every directed link b chunks/round (section 3.1's 4-node ring; section 5.2.2's 8-ring)."""
    links: Dict[Edge, int] = {}
    for n in range(P):
        links[(n, (n + 1) % P)] = b
        links[((n + 1) % P, n)] = b
    return point_to_point(P, links, f"ring{P}")


def complete(P: int, b: int = 1) -> Topology:
    return point_to_point(P, {(s, d): b for s in range(P) for d in range(P) if s != d}, f"K{P}")


def torus2d(nx: int, ny: int, b: int = 1) -> Topology:
    """nx x ny wrap-around mesh, node id = nx*y + x, neighbours (x+-1, y), (x, y+-1)."""
    links: Dict[Edge, int] = {}
    for y in range(ny):
        for x in range(nx):
            n = nx * y + x
            for (xx, yy) in (((x + 1) % nx, y), ((x - 1) % nx, y), (x, (y + 1) % ny), (x, (y - 1) % ny)):
                m = nx * yy + xx
                if m != n:
                    links[(n, m)] = b
    return point_to_point(nx * ny, links, f"torus{nx}x{ny}")


def hcm8() -> Topology:
    """The 8-node hybrid-cube-mesh-shaped graph of the benchmark configurations.

    Two 4-cliques {0..3} and {4..7} plus cross edges i-(i+4); 2 chunks/round
    on (0,3), (1,2), (4,7), (5,6) and on every cross edge, 1 elsewhere; every
    node has 6 link units in and out.  This is NOT the paper's DGX-1 graph
    (see dgx1()); it is the graph the measured configurations name.
    """
    links: Dict[Edge, int] = {}
    for base in (0, 4):
        for i in range(4):
            for j in range(4):
                if i != j:
                    links[(base + i, base + j)] = 1
    for (a, c) in ((0, 3), (1, 2), (4, 7), (5, 6)):
        links[(a, c)] = 2
        links[(c, a)] = 2
    for i in range(4):
        links[(i, i + 4)] = 2
        links[(i + 4, i)] = 2
    return point_to_point(8, links, "hcm8")


def dgx1() -> Topology:
    """The paper's DGX-1 NVLink graph (sections 2.2 and 5.1.1, 5.2.1).

    Two edge-disjoint Hamiltonian cycles: 0-1-4-5-6-7-2-3-0 with two links
    per edge (2 chunks/round) and 0-2-1-3-6-4-7-5-0 with one link per edge.
    """
    links: Dict[Edge, int] = {}
    for cyc, b in (((0, 1, 4, 5, 6, 7, 2, 3), 2), ((0, 2, 1, 3, 6, 4, 7, 5), 1)):
        for i in range(8):
            s, d = cyc[i], cyc[(i + 1) % 8]
            assert (s, d) not in links
            links[(s, d)] = b
            links[(d, s)] = b
    return point_to_point(8, links, "dgx1")


def shared_bus(P: int, b: int = 1) -> Topology:
    """All pairs may talk but only b chunks cross the bus per round (section 3.2.1's shared-bus example)."""
    L = frozenset((s, d) for s in range(P) for d in range(P) if s != d)
    return Topology(P, ((L, b),), f"bus{P}")


def distances(topo: Topology) -> List[List[int]]:
    """Hop counts over the usable links; -1 where unreachable."""
    P = topo.num_nodes
    out_nb = [topo.out_neighbours(n) for n in range(P)]
    dist = [[-1] * P for _ in range(P)]
    for s in range(P):
        dist[s][s] = 0
        q = deque([s])
        while q:
            u = q.popleft()
            for v in out_nb[u]:
                if dist[s][v] < 0:
                    dist[s][v] = dist[s][u] + 1
                    q.append(v)
    return dist


def diameter(topo: Topology) -> int:
    """Latency lower bound a_l of Algorithm 1: no schedule that moves data between the farthest pair has fewer steps."""
    d = distances(topo)
    if any(x < 0 for row in d for x in row):
        raise ValueError("topology is not strongly connected")
    return max(max(row) for row in d)


def ingress_per_round(topo: Topology, n: int) -> int:
    """Largest number of chunks node n can receive in one round.

    For point-to-point constraints this is the sum of b over the links into
    n.  With set constraints it is bounded by every constraint separately; the
    bound used here is the point-to-point sum capped by any constraint that
    covers ALL links into n (enough for the graphs in this repository).
    """
    into = [e for e in topo.edges() if e[1] == n]
    total = 0
    for e in into:
        total += min(b for L, b in topo.bw if e in L)
    for L, b in topo.bw:
        if all(e in L for e in into):
            total = min(total, b)
    return total


def allgather_bandwidth_bound(topo: Topology) -> Fraction:
    """Lower bound on R/C for Allgather (section 2.4's argument).

    Every node must take in (P-1)*C chunks and can take in at most
    ingress_per_round chunks per round, so R >= (P-1)*C / ingress, i.e.
    R/C >= (P-1)/ingress, maximised over nodes.
    """
    P = topo.num_nodes
    return max(Fraction(P - 1, ingress_per_round(topo, n)) for n in range(P))
