"""Pins for oracle/validate.py: the run / validity definitions of section 3.3 and the worked example of section 3.1."""
import numpy as np
import pytest

from conftest import read_examples
from oracle import collective as col
from oracle import generate as gen
from oracle import topology as tp
from oracle.schedule import COPY, REDUCE, Schedule, make_schedule
from oracle.validate import Verdict, run, validate


def test_recursive_doubling_example_of_section_3_1():
    ex = read_examples()
    t, ag = tp.ring(4), col.allgather(4, 1)
    s = gen.recursive_doubling_ring4()
    rep = validate(t, ag, s)
    assert rep.ok, rep.detail
    assert rep.num_steps == int(ex["ring4_recursive_doubling_steps"][0])
    assert rep.num_rounds == int(ex["ring4_recursive_doubling_rounds"][0])
    assert rep.k == 1                                    # the caption calls it 1-synchronous
    assert rep.links_used_per_step == [int(ex["ring4_recursive_doubling_links_per_step"][0])] * 2
    # with one round in the second step the same sends exceed the link bandwidth
    assert validate(t, ag, Schedule([1, 1], s.sends)).verdict is Verdict.BANDWIDTH


def test_run_definition():
    ag = col.allgather(4, 1)
    s = gen.recursive_doubling_ring4()
    V = run(ag, s)
    assert len(V) == 3
    assert (V[0] == ag.pre.astype(bool)).all()
    assert V[1].sum() == 8 and V[2].all()
    for a, b in zip(V, V[1:]):
        assert (b | a == b).all()                        # V only grows
    # a send whose source does not hold the chunk adds nothing to the run
    bogus = make_schedule([1], [(0, 1, 2, 0)])
    assert (run(ag, bogus)[1] == ag.pre.astype(bool)).all()


def _ag3():
    # 3-ring Allgather in one step: every node sends its chunk both ways
    sends = [(n, n, (n + 1) % 3, 0) for n in range(3)] + [(n, n, (n - 1) % 3, 0) for n in range(3)]
    return tp.ring(3), col.allgather(3, 1), make_schedule([1], sends)


def test_valid_tiny_allgather():
    t, ag, s = _ag3()
    assert validate(t, ag, s).ok


def test_one_bad_plan_per_error():
    t, ag, s = _ag3()
    S = lambda rounds, sends: make_schedule(rounds, sends)
    good = s.sends.tolist()
    # out of range chunk / node / step, zero rounds, src == dst, unknown op, REDUCE where nothing combines
    assert validate(t, ag, S([1], [(3, 0, 1, 0)])).verdict is Verdict.INVALID_ARG
    assert validate(t, ag, S([1], [(0, 0, 3, 0)])).verdict is Verdict.INVALID_ARG
    assert validate(t, ag, S([1], [(0, 0, 1, 1)])).verdict is Verdict.INVALID_ARG
    assert validate(t, ag, S([0], good)).verdict is Verdict.INVALID_ARG
    assert validate(t, ag, S([1], [(0, 0, 0, 0)])).verdict is Verdict.INVALID_ARG
    assert validate(t, ag, S([1], [(0, 0, 1, 0, 7)])).verdict is Verdict.INVALID_ARG
    assert validate(t, ag, S([1], [(0, 0, 1, 0, REDUCE)])).verdict is Verdict.INVALID_ARG
    assert validate(tp.ring(4), ag, s).verdict is Verdict.INVALID_ARG
    # no link 0 -> 2 on the 4-ring
    assert validate(tp.ring(4), col.allgather(4, 1), S([1], [(0, 0, 2, 0)])).verdict is Verdict.SEND_NO_LINK
    # node 1 does not hold chunk 0 at step 0
    assert validate(t, ag, S([1], [(0, 1, 2, 0)])).verdict is Verdict.SEND_NO_SOURCE
    # chunk forwarded in the step it arrives: the source is not in V_s yet
    assert validate(tp.ring(4), col.allgather(4, 1),
                    S([1], [(0, 0, 1, 0), (0, 1, 2, 0)])).verdict is Verdict.SEND_NO_SOURCE
    # two chunks over a one-chunk link in a one-round step
    ag2 = col.allgather(3, 2)
    assert validate(t, ag2, S([1], [(0, 0, 1, 0), (3, 0, 1, 0)])).verdict is Verdict.BANDWIDTH
    assert validate(t, ag2, S([2], [(0, 0, 1, 0), (3, 0, 1, 0)])).verdict is Verdict.POSTCONDITION
    # post not reached
    assert validate(t, ag, S([1], good[:-1])).verdict is Verdict.POSTCONDITION
    # the same (chunk, node) written by two sends of one step
    k4 = tp.complete(4)
    bc = col.broadcast(4, 1, root=0)
    assert validate(k4, bc, S([1, 1], [(0, 0, 1, 0), (0, 0, 2, 0), (0, 1, 3, 1), (0, 2, 3, 1)])).verdict is Verdict.HAZARD


def test_shared_constraint_counts_all_its_edges():
    bus = tp.shared_bus(3)
    ag = col.allgather(3, 1)
    sends = [(n, n, (n + 1) % 3, 0) for n in range(3)] + [(n, n, (n - 1) % 3, 0) for n in range(3)]
    assert validate(bus, ag, make_schedule([1], sends)).verdict is Verdict.BANDWIDTH
    assert validate(bus, ag, make_schedule([6], sends)).ok       # six rounds of one chunk each


def test_combining_rules():
    t = tp.ring(3)
    ar = col.allreduce(3, 1)
    R, C = REDUCE, COPY
    # chain 2 -> 1 -> 0 then broadcast back 0 -> 1, 0 -> 2
    ok = make_schedule([1, 1, 1], [(0, 2, 1, 0, R), (0, 1, 0, 1, R), (0, 0, 1, 2, C), (0, 0, 2, 2, C)])
    assert validate(t, ar, ok).ok
    # read and written in the same step
    bad = make_schedule([1, 1], [(0, 2, 1, 0, R), (0, 1, 0, 0, R), (0, 0, 1, 1, C), (0, 0, 2, 1, C)])
    assert validate(t, ar, bad).verdict is Verdict.HAZARD
    # rank 2 counted twice: it is sent to both 0 and 1, and 1 is then folded into 0
    twice = make_schedule([1, 1, 1], [(0, 2, 1, 0, R), (0, 2, 0, 0, R), (0, 1, 0, 1, R), (0, 0, 1, 2, C), (0, 0, 2, 2, C)])
    assert validate(t, ar, twice).verdict is Verdict.HAZARD
    # a consumed partial is read again
    again = make_schedule([1, 1, 1], [(0, 2, 1, 0, R), (0, 2, 0, 1, R), (0, 1, 0, 2, R)])
    assert validate(t, ar, again).verdict is Verdict.SEND_NO_SOURCE
    # incomplete sum copied everywhere
    short = make_schedule([1, 1], [(0, 1, 0, 0, R), (0, 0, 1, 1, C), (0, 0, 2, 1, C)])
    assert validate(t, ar, short).verdict is Verdict.POSTCONDITION
    # Reducescatter only needs the owner complete
    rs = col.reducescatter(3, 3)
    sends = []
    for c in range(3):
        sends += [(c, (c + 2) % 3, (c + 1) % 3, 0, R), (c, (c + 1) % 3, c, 1, R)]
    assert validate(t, rs, make_schedule([1, 1], sends)).ok
    # copy and reduce into one (chunk, node) in the same step
    mixed = make_schedule([1], [(0, 1, 0, 0, C), (0, 2, 0, 0, R)])
    assert validate(t, ar, mixed).verdict is Verdict.HAZARD
