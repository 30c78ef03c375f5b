"""Every row of the paper's Tables 4 and 5, pinned by a stored witness.

tests/golden/witnesses/ holds one schedule per non-Allreduce row, found by the exact search
(`python -m oracle.reproduce_tables --write`; the largest took minutes, which is why they are stored).  Here each is
read back and checked from scratch by the validator (seconds): it is valid on its topology, has the row's S and R,
reaches the collective's post-condition, and respects every link's bandwidth in every round; the library's own
validator must agree.  Every Allreduce row is the row of the table whose Allgather it is composed from (section
3.5): (P*C, 2S, 2R).  tests/golden/reproduced_rows.txt records the verdicts of the search, including the
infeasibility of one step fewer (latency-optimal rows) and one round fewer (bandwidth-optimal rows).
"""
import os

import pytest

from conftest import GOLDEN, read_table
from helpers import plan_status
from oracle import collective as col
from oracle import generate as gen
from oracle import reproduce_tables as rt
from oracle import topology as tp
from oracle.validate import validate

TABLES = [("table5_z52.txt", "ring8", tp.ring(8)), ("table4_dgx1.txt", "dgx1", tp.dgx1())]
ROWS = [(tname, topo, r) for table, tname, topo in TABLES for r in read_table(table)]


def reproduced():
    out = {}
    with open(os.path.join(GOLDEN, "reproduced_rows.txt")) as f:
        for line in f:
            line = line.split("#")[0].split()
            if line:
                out[(line[0], line[1], int(line[2]), int(line[3]), int(line[4]))] = line[5:]
    return out


@pytest.mark.parametrize("tname,topo,row", [r for r in ROWS if r[2][0] != "allreduce"],
                         ids=[f"{r[0]}-{r[2][0]}-{r[2][1]}-{r[2][2]}-{r[2][3]}" for r in ROWS if r[2][0] != "allreduce"])
def test_stored_witness_is_a_valid_schedule_with_the_rows_steps_and_rounds(tname, topo, row):
    name, C, S, R, a, b, opt = row
    sched = rt.read_witness(rt.witness_path(tname, name, C, S, R))
    coll = rt.MAKE[name](8, C)
    rep = validate(topo, coll, sched)
    assert rep.ok, rep.detail
    assert (sched.num_steps, sched.num_rounds) == (S, R) and (sched.sends[:, 4] == 0).all()
    assert a == S and b * C == R                                       # the running time the table prints: S alpha + R/C L beta
    status, st = plan_status(topo, coll, sched, "f32", 8)              # the library's validator, independently written
    assert status == "SCCL_OK" and (st["num_steps"], st["num_rounds"], st["k"]) == (S, R, R - S)
    opt_rec, verdict, fewer_steps, fewer_rounds = reproduced()[(tname, name, C, S, R)]
    assert verdict == "feasible" and opt_rec == opt
    if opt in ("latency", "both") and S > 1:
        assert fewer_steps == "infeasible"
    if opt in ("bandwidth", "both") and R > S:
        assert fewer_rounds == "infeasible"


@pytest.mark.parametrize("tname,topo,row", [r for r in ROWS if r[2][0] == "allreduce"],
                         ids=[f"{r[0]}-{r[2][0]}-{r[2][1]}-{r[2][2]}-{r[2][3]}" for r in ROWS if r[2][0] == "allreduce"])
def test_allreduce_rows_are_the_allgather_witnesses_composed_with_their_inverse(tname, topo, row):
    _, C, S, R, a, b, opt = row
    assert C % 8 == 0 and S % 2 == 0 and R % 2 == 0
    ag = col.allgather(8, C // 8)
    base = rt.read_witness(rt.witness_path(tname, "allgather", C // 8, S // 2, R // 2))
    ar, arc = gen.compose_allreduce(base, ag)
    assert validate(topo, arc, ar).ok
    assert ar.csr(arc.num_chunks) == (C, S, R)
    status, st = plan_status(topo, arc, ar, "f16", 8)
    assert status == "SCCL_OK" and (st["num_steps"], st["num_rounds"]) == (S, R)
