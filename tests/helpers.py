"""Test glue: turns the oracle's descriptions into the binding's (plain data; no arithmetic of the method)."""
import numpy as np

from paper_2008_08708_amd import sccl

VERDICT_TO_STATUS = {
    "OK": "SCCL_OK", "INVALID_ARG": "SCCL_ERR_INVALID_ARG", "SEND_NO_LINK": "SCCL_ERR_SEND_NO_LINK",
    "SEND_NO_SOURCE": "SCCL_ERR_SEND_NO_SOURCE", "BANDWIDTH": "SCCL_ERR_BANDWIDTH", "HAZARD": "SCCL_ERR_HAZARD",
    "POSTCONDITION": "SCCL_ERR_POSTCONDITION",
}


def to_binding(topo, coll, sched, dtype, elems_per_chunk, slot=None, slots_per_rank=0):
    t = sccl.Topology(topo.num_nodes, [(sorted(L), b) for (L, b) in topo.bw])
    c = sccl.Collective(coll.num_chunks, coll.pre, coll.post, coll.combining, dtype, elems_per_chunk, slot, slots_per_rank)
    s = sccl.Schedule(list(sched.rounds), np.asarray(sched.sends, dtype=np.int32))
    return t, c, s


def plan_status(topo, coll, sched, dtype="f32", elems_per_chunk=4, options=None, slot=None, slots_per_rank=0):
    """Status name sccl_plan_create_ex returns for a host-only plan."""
    opts = {"flags": sccl.SCCL_PLAN_HOST_ONLY}
    opts.update(options or {})
    try:
        p = sccl.sccl_plan_create(*to_binding(topo, coll, sched, dtype, elems_per_chunk, slot, slots_per_rank), options=opts)
    except sccl.ScclError as e:
        return e.name, None
    st = sccl.sccl_plan_stats(p)
    sccl.sccl_plan_destroy(p)
    return "SCCL_OK", st
