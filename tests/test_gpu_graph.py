"""sccl_execute under HIP graph capture: the call only checks pointers on the host and enqueues one kernel (no
allocation, no memset, no synchronisation), so it can be recorded into a graph and replayed.  Every replay is
compared with the oracle, with eager work and synchronisations between the replays."""
import numpy as np
import pytest

from gpu_util import assert_same_bits, host_inputs
from helpers import to_binding
from oracle import collective as col
from oracle import executor as ex
from oracle import generate as gen
from oracle import topology as tp
from paper_2008_08708_amd import sccl

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("lowering", [sccl.SCCL_LOWER_MEMORY, sccl.SCCL_LOWER_STAGED])
@pytest.mark.parametrize("epc", [4, 4 * 1031])
def test_graph_replays_equal_the_oracle(lowering, epc):
    import torch
    topo = tp.torus2d(4, 4)
    ag = col.allgather(16, 2)
    sched, coll = gen.compose_allreduce(gen.greedy_bfs(topo, ag), ag)
    P, G = 16, coll.num_chunks
    plan = sccl.sccl_plan_create(*to_binding(topo, coll, sched, "f32", epc), options={"lowering": lowering})
    pristine = [torch.empty(G * epc, dtype=torch.float32, device="cuda") for _ in range(P)]
    work = [torch.empty_like(p) for p in pristine]
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    print(f"[case] graph capture lowering={lowering} epc={epc}", flush=True)
    for p in pristine:
        p.zero_()
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        for w, p in zip(work, pristine):
            w.copy_(p)                                     # restore, then the collective, both inside the graph
        sccl.sccl_execute(plan, work, side)
    for seed in (5, 6, 7):
        bufs = host_inputs("uniform", "f32", seed, P, G, epc)
        want = [b.copy() for b in bufs]
        ex.execute("f32", G, epc, sched, want)
        for p, b in zip(pristine, bufs):                   # eager work between the replays
            p.copy_(torch.from_numpy(b))
        torch.cuda.synchronize()
        print(f"[case]   replay seed={seed}", flush=True)
        graph.replay()
        torch.cuda.synchronize()
        assert_same_bits(want, [w.cpu().numpy() for w in work])
        eager = [p.clone() for p in pristine]
        sccl.sccl_execute(plan, eager)
        torch.cuda.synchronize()
        for e, w in zip(eager, work):
            assert torch.equal(e.view(torch.int32), w.view(torch.int32))
    del graph
    sccl.sccl_plan_destroy(plan)


@pytest.mark.parametrize("lowering", [sccl.SCCL_LOWER_MEMORY, sccl.SCCL_LOWER_STAGED])
def test_one_plan_on_two_streams_with_different_buffers(lowering):
    """A plan holds no mutable state: two executes of it may run at the same time on two (default-priority) streams
    as long as their rank buffers differ."""
    import torch
    topo = tp.hcm8()
    ag = col.allgather(8, 2)
    sched, coll = gen.compose_allreduce(gen.greedy_bfs(topo, ag), ag)
    P, G, epc = 8, coll.num_chunks, 4 * 4099
    plan = sccl.sccl_plan_create(*to_binding(topo, coll, sched, "f32", epc), options={"lowering": lowering})
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    sets, wants = [], []
    for seed in (11, 12):
        bufs = host_inputs("uniform", "f32", seed, P, G, epc)
        want = [b.copy() for b in bufs]
        ex.execute("f32", G, epc, sched, want)
        wants.append(want)
        sets.append([torch.from_numpy(b).cuda() for b in bufs])
    torch.cuda.synchronize()
    print(f"[case] two streams lowering={lowering}", flush=True)
    for st, dev in zip(streams, sets):                      # back to back: the two kernels overlap on the device
        sccl.sccl_execute(plan, dev, st)
    torch.cuda.synchronize()
    for dev, want in zip(sets, wants):
        assert_same_bits(want, [d.cpu().numpy() for d in dev])
    sccl.sccl_plan_destroy(plan)
