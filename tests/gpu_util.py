"""Helpers of the GPU parity tests: run one case on both sides and compare bits."""
import numpy as np

from helpers import to_binding
from oracle import executor as ex
from paper_2008_08708_amd import inputs, sccl

NP = {"i32": np.int32, "f32": np.float32, "f16": np.float16}


def bits(a):
    return a.view(np.uint32 if a.dtype.itemsize == 4 else np.uint16)


def host_inputs(dist, dtype, seed, P, G, epc, pre=None):
    bufs = [inputs.generate(dist, dtype, seed, n, 0, G * epc) for n in range(P)]
    if pre is not None:
        for n in range(P):
            for c in range(G):
                if not pre[c, n]:
                    inputs.poison(bufs[n], c * epc, (c + 1) * epc)
    return bufs


def run_both(topo, coll, sched, dtype, bufs, epc, options=None, label="", mode="sccl_execute", slot=None, slots_per_rank=0):
    """Oracle on copies of `bufs`, library on device copies; returns (oracle buffers, gpu buffers as numpy)."""
    import torch
    print(f"[case] {label} {mode} P={coll.num_nodes} G={coll.num_chunks} epc={epc} dtype={dtype} opts={options}", flush=True)
    want = [b.copy() for b in bufs]
    ex.execute(dtype, coll.num_chunks, epc, sched, want, slot=slot, slots_per_rank=slots_per_rank)
    dev = [torch.from_numpy(b.copy()).cuda() for b in bufs]
    plan = sccl.sccl_plan_create(*to_binding(topo, coll, sched, dtype, epc, slot, slots_per_rank), options=options)
    getattr(sccl, mode)(plan, dev)
    torch.cuda.synchronize()
    got = [d.cpu().numpy() for d in dev]
    sccl.sccl_plan_destroy(plan)
    return want, got


def assert_same_bits(want, got):
    for n, (w, g) in enumerate(zip(want, got)):
        bad = np.nonzero(bits(w) != bits(g))[0]
        assert bad.size == 0, f"rank {n}: {bad.size} elements differ, first at {bad[0]}: want {w[bad[0]]!r} got {g[bad[0]]!r}"
