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
    """Oracle on copies of `bufs`, library on device copies; returns (oracle buffers, gpu buffers as numpy).

    sccl_execute has two lowerings (through memory, staged in the local data share).  Unless `options` names
    one, the case runs under BOTH -- the staged one whenever the plan says it is available -- each is compared
    with the oracle here, and the through-memory result is returned."""
    import torch
    want = [b.copy() for b in bufs]
    ex.execute(dtype, coll.num_chunks, epc, sched, want, slot=slot, slots_per_rank=slots_per_rank)
    args = to_binding(topo, coll, sched, dtype, epc, slot, slots_per_rank)
    explicit = mode != "sccl_execute" or (options is not None and options.get("lowering", 0) != 0)
    lowerings = [None] if explicit else [sccl.SCCL_LOWER_MEMORY, sccl.SCCL_LOWER_STAGED]
    result = None
    for low in lowerings:
        opts = dict(options or {})
        if low is not None:
            opts["lowering"] = low
        print(f"[case] {label} {mode} P={coll.num_nodes} G={coll.num_chunks} epc={epc} dtype={dtype} opts={opts}", flush=True)
        try:
            plan = sccl.sccl_plan_create(*args, options=opts or None)
        except sccl.ScclError as e:
            if low == sccl.SCCL_LOWER_STAGED and e.name == "SCCL_ERR_INVALID_ARG":
                print("[case]   staged lowering not available for this plan", flush=True)
                continue
            raise
        dev = [torch.from_numpy(b.copy()).cuda() for b in bufs]
        getattr(sccl, mode)(plan, dev)
        torch.cuda.synchronize()
        got = [d.cpu().numpy() for d in dev]
        sccl.sccl_plan_destroy(plan)
        if result is None:
            result = got
        else:
            assert_same_bits(want, got)
    return want, result


def assert_same_bits(want, got):
    for n, (w, g) in enumerate(zip(want, got)):
        bad = np.nonzero(bits(w) != bits(g))[0]
        assert bad.size == 0, f"rank {n}: {bad.size} elements differ, first at {bad[0]}: want {w[bad[0]]!r} got {g[bad[0]]!r}"
