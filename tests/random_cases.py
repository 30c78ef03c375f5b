"""Seeded random topologies and schedules for robustness tests (plain data; built with the oracle's generators)."""
import numpy as np

from oracle import collective as col
from oracle import generate as gen
from oracle import topology as tp


def random_symmetric_topology(rng, P):
    """A connected undirected graph on P nodes (random spanning tree plus random extra edges), b in {1, 2, 3}."""
    links = {}
    order = rng.permutation(P).tolist()
    for i in range(1, P):
        a, b = order[i], order[int(rng.integers(0, i))]
        w = int(rng.integers(1, 4))
        links[(a, b)] = w
        links[(b, a)] = w
    for _ in range(int(rng.integers(0, 2 * P))):
        a, b = int(rng.integers(0, P)), int(rng.integers(0, P))
        if a != b and (a, b) not in links:
            w = int(rng.integers(1, 4))
            links[(a, b)] = w
            links[(b, a)] = w
    return tp.point_to_point(P, links, f"rand{P}")


def random_case(seed):
    """(label, topology, collective, schedule, dtype, distribution, elems_per_chunk)"""
    rng = np.random.default_rng(seed)
    P = int(rng.integers(2, 13))
    topo = random_symmetric_topology(rng, P)
    C = int(rng.integers(1, 4))
    what = ["allgather", "allreduce", "reducescatter", "broadcast", "alltoall", "gather"][int(rng.integers(0, 6))]
    dtype, dist = [("f32", "uniform"), ("f16", "normal"), ("i32", "u32")][int(rng.integers(0, 3))]
    if dtype == "f32" and seed % 2:
        dist = "wide"                                           # sums that round: the order of additions shows in the bits
    epc = int([1, 3, 16, 257, 1024, 2048 + 4 * int(rng.integers(0, 64)), 3 * 4096 + 8 * int(rng.integers(0, 64))][int(rng.integers(0, 7))])
    ag = col.allgather(P, C)
    rounds = [int(rng.integers(1, 3)) for _ in range(4)]        # some steps get two rounds
    if what in ("allgather", "allreduce", "reducescatter"):
        base = gen.greedy_bfs(topo, ag, rounds=rounds)
        if what == "allgather":
            coll, sched = ag, base
        elif what == "allreduce":
            sched, coll = gen.compose_allreduce(base, ag)
        else:
            sched, coll = gen.reducescatter_from(base, ag)
    else:
        coll = {"broadcast": lambda: col.broadcast(P, C, int(rng.integers(0, P))),
                "alltoall": lambda: col.alltoall(P, P),
                "gather": lambda: col.gather(P, C, int(rng.integers(0, P)))}[what]()
        sched = gen.greedy_route(topo, coll, rounds=rounds)
    return f"seed{seed}-{what}-P{P}-C{C}-{dtype}-{epc}", topo, coll, sched, dtype, dist, epc
