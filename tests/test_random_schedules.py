"""Randomised robustness: random connected topologies, collectives, chunk counts, rounds, element types and sizes.
CPU: the generators' output validates, the library's host validation agrees, the oracle's result has the closed
form.  GPU: bit-exact parity."""
import numpy as np
import pytest

from gpu_util import assert_same_bits, run_both
from helpers import plan_status
from oracle import executor as ex
from oracle.validate import validate
from paper_2008_08708_amd import inputs
from random_cases import random_case

import os

# 40 seeds by default; SCCL_MORE_SEEDS=N adds seeds 1000 .. 1000+N-1 for a longer soak of the same tests
SEEDS = list(range(100, 140)) + list(range(1000, 1000 + int(os.environ.get("SCCL_MORE_SEEDS", "0"))))


def make_inputs(coll, dtype, dist, seed, epc):
    bufs = [inputs.generate(dist, dtype, seed, n, 0, coll.num_chunks * epc) for n in range(coll.num_nodes)]
    if not coll.combining:
        for n in range(coll.num_nodes):
            for c in range(coll.num_chunks):
                if not coll.pre[c, n]:
                    inputs.poison(bufs[n], c * epc, (c + 1) * epc)
    return bufs


@pytest.mark.parametrize("seed", SEEDS)
def test_random_case_validates_and_has_the_closed_form(seed):
    label, topo, coll, sched, dtype, dist, epc = random_case(seed)
    rep = validate(topo, coll, sched)
    assert rep.ok, (label, rep.detail)
    name, st = plan_status(topo, coll, sched, dtype, epc)
    assert name == "SCCL_OK", label
    assert st["bytes_min"] == ex.algorithmic_bytes(sched, epc * (2 if dtype == "f16" else 4))[0]
    epc = min(epc, 64)                                       # the closed-form check does not need the full size
    if coll.combining and dtype != "i32":
        dist = "smallint"                                    # exact in any order
    bufs = make_inputs(coll, dtype, dist, seed, epc)
    pristine = [b.copy() for b in bufs]
    ex.execute(dtype, coll.num_chunks, epc, sched, bufs)
    P, G = coll.num_nodes, coll.num_chunks
    if coll.combining:
        if dtype == "i32":
            total = np.zeros(G * epc, dtype=np.uint32)
            for b in pristine:
                total = total + b.view(np.uint32)
            got = lambda n: bufs[n].view(np.uint32)
        else:
            total = sum(b.astype(np.float64) for b in pristine)
            got = lambda n: bufs[n].astype(np.float64)
        for c in range(G):
            for n in range(P):
                if coll.post[c, n]:
                    assert (got(n)[c * epc:(c + 1) * epc] == total[c * epc:(c + 1) * epc]).all(), label
    else:
        u = np.uint32 if bufs[0].dtype.itemsize == 4 else np.uint16
        for c in range(G):
            owner = int(np.nonzero(coll.pre[c])[0][0])
            for n in range(P):
                if coll.post[c, n]:
                    assert (bufs[n].view(u)[c * epc:(c + 1) * epc] == pristine[owner].view(u)[c * epc:(c + 1) * epc]).all(), label


@pytest.mark.parametrize("seed", SEEDS)
def test_mutated_random_case_gets_the_oracles_verdict(seed):
    """Break a valid random schedule in one place (a send's field, a dropped or repeated send, a step's rounds, a
    bit of post): the library's host validation and the oracle's validator must name the same defect, or both accept."""
    from helpers import VERDICT_TO_STATUS
    from oracle.schedule import Schedule
    from oracle.collective import Collective
    label, topo, coll, sched, dtype, dist, epc = random_case(seed)
    rng = np.random.default_rng(seed + 77)
    P, G, S = coll.num_nodes, coll.num_chunks, sched.num_steps
    for trial in range(12):
        sends, rounds, post = sched.sends.copy(), list(sched.rounds), coll.post.copy()
        kind = int(rng.integers(0, 6))
        n = sends.shape[0]
        if kind == 0 and n:
            i, f = int(rng.integers(0, n)), int(rng.integers(0, 5))
            hi = (G, P, P, S, 2)[f]
            sends[i, f] = int(rng.integers(-1, hi + 1))
        elif kind == 1 and n:
            sends = np.delete(sends, int(rng.integers(0, n)), axis=0)
        elif kind == 2 and n:
            i = int(rng.integers(0, n))
            sends = np.insert(sends, i, sends[i], axis=0)
        elif kind == 3:
            rounds[int(rng.integers(0, S))] = int(rng.integers(0, 3))
        elif kind == 4:
            post[int(rng.integers(0, G)), int(rng.integers(0, P))] ^= 1
        elif kind == 5 and n > 1:
            i, j = rng.integers(0, n, size=2)
            sends[[i, j], 3] = sends[[j, i], 3]                 # two sends trade steps
        m = Schedule(rounds, sends)
        c = Collective(coll.name, P, G, coll.pre, post, coll.combining, coll.chunks_per_node)
        want = VERDICT_TO_STATUS[validate(topo, c, m).verdict.value]
        got, _ = plan_status(topo, c, m, dtype, 4)
        assert got == want, (label, trial, kind)


@pytest.mark.gpu
@pytest.mark.parametrize("seed", SEEDS)
@pytest.mark.parametrize("mode", ["sccl_execute", "sccl_execute_stepwise"])
def test_random_case_gpu_parity(seed, mode):
    label, topo, coll, sched, dtype, dist, epc = random_case(seed)
    bufs = make_inputs(coll, dtype, dist, seed, epc)
    want, got = run_both(topo, coll, sched, dtype, bufs, epc, label=label, mode=mode)
    assert_same_bits(want, got)
