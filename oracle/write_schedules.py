"""Writes the schedule files of the five benchmark configurations (calls only oracle/ code).

Run from the repository root:  python -m oracle.write_schedules
The files land in paper_2008_08708_amd/schedules/ and are what the benchmark
feeds to the GPU library; tests check that they are exactly what this script
writes and that the oracle's validator accepts them.
"""
from __future__ import annotations

import os
import sys

import numpy as np

from . import collective as col
from . import generate as gen
from . import topology as tp
from .validate import validate

OUT = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2008_08708_amd", "schedules")


def _rel_word(rel, G, P):
    if rel.all():
        return "all", []
    if (rel == col.rel_scattered(G, P)).all():
        return "scattered", []
    if (rel == col.rel_transpose(G, P)).all():
        return "transpose", []
    for n in range(P):
        if (rel == col.rel_root(G, P, n)).all():
            return f"root:{n}", []
    return "rows", ["".join(str(int(x)) for x in row) for row in rel]


def render(name, topo, coll, sched, slot=None, slots_per_rank=0) -> str:
    rep = validate(topo, coll, sched)
    if not rep.ok:
        raise RuntimeError(f"{name}: {rep.verdict} {rep.detail}")
    P, G = coll.num_nodes, coll.num_chunks
    out = ["sccl-schedule 1", f"name {name}", f"collective {coll.name} combining {int(coll.combining)}",
           f"nodes {P}", f"chunks {G}", f"chunks_per_node {coll.chunks_per_node}"]
    for key, rel in (("pre", coll.pre), ("post", coll.post)):
        word, rows = _rel_word(rel, G, P)
        out.append(f"{key} {word}")
        out += rows
    for L, b in topo.bw:
        out.append(f"bw {b} " + " ".join(f"{s}>{d}" for (s, d) in sorted(L)))
    if slot is not None:
        out.append(f"slots {int(slots_per_rank)}")
        out += [" ".join(str(int(x)) for x in row) for row in np.asarray(slot).tolist()]
    out.append("rounds " + " ".join(str(r) for r in sched.rounds))
    out.append(f"sends {sched.sends.shape[0]}")
    out += [" ".join(str(int(x)) for x in row) for row in sched.sends.tolist()]
    return "\n".join(out) + "\n"


def configurations():
    """name -> (topology, collective, schedule) for the five configurations."""
    out = {}
    # 1: Allgather, 4-ring, one chunk per node, greedy (2 steps)
    t = tp.ring(4)
    ag = col.allgather(4, 1)
    out["cfg1_allgather_ring4"] = (t, ag, gen.greedy_bfs(t, ag))
    # 2: Allgather, 8-node graph, two chunks per node
    t = tp.hcm8()
    ag = col.allgather(8, 2)
    out["cfg2_allgather_hcm8"] = (t, ag, gen.greedy_bfs(t, ag))
    # 3: Allreduce on the same graph, 8 chunks per rank = inverse(Allgather C=1) ; Allgather
    ag = col.allgather(8, 1)
    ar, arc = gen.compose_allreduce(gen.greedy_bfs(t, ag), ag)
    out["cfg3_allreduce_hcm8"] = (t, arc, ar)
    # 4: ring Allreduce on the 8-ring, two chunks per rank per direction (C = 4, 14 steps of 2 rounds)
    t = tp.ring(8)
    ag = col.allgather(8, 4)
    ar, arc = gen.compose_allreduce(gen.ring_allgather(8, 4), ag)
    out["cfg4_allreduce_ring8"] = (t, arc, ar)
    #    and the paper's own row for that machine: C = 2, (16, 14, 14)
    ag = col.allgather(8, 2)
    ar, arc = gen.compose_allreduce(gen.ring_allgather(8, 2), ag)
    out["cfg4b_allreduce_ring8_c2"] = (t, arc, ar)
    # 5: 4x4 torus, four chunks per node, Allgather and Allreduce
    t = tp.torus2d(4, 4)
    ag = col.allgather(16, 4)
    s = gen.greedy_bfs(t, ag)
    out["cfg5_allgather_torus4x4"] = (t, ag, s)
    ar, arc = gen.compose_allreduce(s, ag)
    out["cfg5_allreduce_torus4x4"] = (t, arc, ar)
    #    and the latency-optimal algorithm for the same topology, from the exact search: one chunk per node,
    #    (C, S, R) = (1, 4, 4) with S the diameter; Allreduce (16, 8, 8).  The pair the cost model chooses between.
    from . import synthesize as syn
    ag = col.allgather(16, 1)
    s = syn.solve_instance(t, ag, 4, 4)
    out["cfg5_allgather_torus4x4_latency"] = (t, ag, s)
    ar, arc = gen.compose_allreduce(s, ag)
    out["cfg5_allreduce_torus4x4_latency"] = (t, arc, ar)
    return out


def layouts():
    """name -> (slot map, chunks per rank buffer) for the configurations that do not keep chunk c at position c."""
    cfg = extra_configurations()
    t, a2a, s = cfg["alltoall_dgx1"]
    return {"alltoall_dgx1": col.compact_slots(a2a, s.sends)}


def extra_configurations():
    """Schedules beyond the five configurations: the collective the paper gains most on (section 5.5.3), on its
    own topology.  Alltoall on the DGX-1 graph, eight chunks per node (one per destination): the row (8, 3, 3)
    of Table 4, found again by the exact search."""
    from . import synthesize as syn
    t = tp.dgx1()
    a2a = col.alltoall(8, 8)
    out = {"alltoall_dgx1": (t, a2a, syn.solve_instance(t, a2a, 3, 3))}
    # the remaining collectives of Table 2, and Reduce by inversion (section 3.5), on the same graph: the
    # latency-optimal rows the shortest-path generator reaches (Broadcast (2,2,2), Gather (1,2,2))
    bc = col.broadcast(8, 2, 0)
    s_bc = gen.greedy_route(t, bc)
    out["broadcast_dgx1"] = (t, bc, s_bc)
    out["reduce_dgx1"] = (t.reversed(), col.reduce(8, 2, 0), gen.invert(s_bc, bc))
    ga = col.gather(8, 1, 0)
    out["gather_dgx1"] = (t, ga, gen.greedy_route(t, ga))
    sc = col.scatter(8, 8, 0)
    out["scatter_dgx1"] = (t, sc, gen.greedy_route(t, sc))
    # Reducescatter, the inverse of an Allgather (section 3.5): the paper's DGX-1 Allgather row (2,3,3) inverted,
    # (16,3,3) in its Table 4 footnote's counting (C times 8), on the reversed graph (the same graph: it is symmetric)
    ag = col.allgather(8, 2)
    rs, rsc = gen.reducescatter_from(syn.solve_instance(t, ag, 3, 3), ag)
    out["reducescatter_dgx1"] = (t.reversed(), rsc, rs)
    return out


def main():
    os.makedirs(OUT, exist_ok=True)
    every = dict(configurations())
    every.update(extra_configurations())
    lay = layouts()
    for name, (topo, coll, sched) in every.items():
        with open(os.path.join(OUT, name + ".txt"), "w") as f:
            f.write(render(name, topo, coll, sched, *lay.get(name, (None, 0))))
        print(name, coll.name, "P", coll.num_nodes, "G", coll.num_chunks, "S", sched.num_steps, "R", sched.num_rounds,
              "sends", sched.sends.shape[0])


if __name__ == "__main__":
    main()
