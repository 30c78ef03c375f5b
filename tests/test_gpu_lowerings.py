"""GPU parity of the two comparator lowerings (one kernel per step; one device copy per send)."""
import numpy as np
import pytest

from gpu_util import assert_same_bits, host_inputs, run_both
from helpers import to_binding
from oracle import collective as col
from oracle import generate as gen
from oracle import topology as tp
from paper_2008_08708_amd import sccl

pytestmark = pytest.mark.gpu

CASES = [
    ("ag-hcm8", tp.hcm8(), 2, "allgather", "greedy", "i32", "u32", 3 * 2048 + 4 * 37),
    ("ag-w4", tp.hcm8(), 2, "allgather", "greedy", "i32", "u32", 1031),
    ("ar-hcm8", tp.hcm8(), 1, "allreduce", "greedy", "f32", "uniform", 5 * 2048 + 4 * 101),
    ("ar-ring-f16", tp.ring(8), 4, "allreduce", "ring", "f16", "normal", 3 * 4096 + 8 * 77),
    ("ar-torus", tp.torus2d(4, 4), 4, "allreduce", "greedy", "f32", "uniform", 2048 + 4 * 3),
    ("ar-tiny", tp.torus2d(4, 4), 4, "allreduce", "greedy", "f32", "uniform", 4),
    ("ar-K12", tp.complete(12), 1, "allreduce", "greedy", "f16", "normal", 1024 + 8),
    ("ag-torus", tp.torus2d(4, 4), 4, "allgather", "greedy", "f32", "uniform", 2048 + 4 * 3),
]


def build(topo, C, what, kind):
    P = topo.num_nodes
    ag = col.allgather(P, C)
    base = gen.ring_allgather(P, C) if kind == "ring" else gen.greedy_bfs(topo, ag)
    if what == "allgather":
        return ag, base, ag.pre
    sched, coll = gen.compose_allreduce(base, ag)
    return coll, sched, None


@pytest.mark.parametrize("label,topo,C,what,kind,dtype,dist,epc", CASES, ids=[c[0] for c in CASES])
def test_stepwise_lowering_bitwise(label, topo, C, what, kind, dtype, dist, epc):
    coll, sched, pre = build(topo, C, what, kind)
    bufs = host_inputs(dist, dtype, 51, topo.num_nodes, coll.num_chunks, epc, pre)
    want, got = run_both(topo, coll, sched, dtype, bufs, epc, label=label, mode="sccl_execute_stepwise")
    assert_same_bits(want, got)


@pytest.mark.parametrize("label,topo,C,what,kind,dtype,dist,epc", [c for c in CASES if c[3] == "allgather"],
                         ids=[c[0] for c in CASES if c[3] == "allgather"])
def test_memcpy_lowering_bitwise(label, topo, C, what, kind, dtype, dist, epc):
    coll, sched, pre = build(topo, C, what, kind)
    bufs = host_inputs(dist, dtype, 53, topo.num_nodes, coll.num_chunks, epc, pre)
    want, got = run_both(topo, coll, sched, dtype, bufs, epc, label=label, mode="sccl_execute_memcpy")
    assert_same_bits(want, got)


def test_memcpy_lowering_refuses_reductions_and_checks_buffers():
    import torch
    topo = tp.hcm8()
    coll, sched, _ = build(topo, 1, "allreduce", "greedy")
    print("[case] memcpy lowering error paths", flush=True)
    plan = sccl.sccl_plan_create(*to_binding(topo, coll, sched, "f32", 16))
    bufs = [torch.zeros(8 * 16, dtype=torch.float32, device="cuda") for _ in range(8)]
    with pytest.raises(sccl.ScclError) as e:
        sccl.sccl_execute_memcpy(plan, bufs)
    assert e.value.name == "SCCL_ERR_INVALID_ARG"
    with pytest.raises(sccl.ScclError) as e:
        sccl.sccl_execute_stepwise(plan, [bufs[0]] * 8)
    assert e.value.name == "SCCL_ERR_OVERLAP"
    sccl.sccl_execute_stepwise(plan, bufs)
    torch.cuda.synchronize()
    sccl.sccl_plan_destroy(plan)
