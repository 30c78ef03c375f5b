"""Re-derives the (C, S, R) rows of the paper's Tables 4 and 5 with the exact search (calls only oracle/ code).

Run from the repository root:
    python -m oracle.reproduce_tables [seconds per instance]            report only
    python -m oracle.reproduce_tables --write [seconds per instance]    also store what was found under tests/golden/

For every row it reports whether a schedule with those S and R was found (and validated) and how long the
solver took; for rows marked latency / bandwidth optimal it also asks for the instance one step / one round
cheaper, which must be infeasible.  With --write every witness schedule goes to
tests/golden/witnesses/<topology>_<collective>_<C>_<S>_<R>.txt and the verdicts to
tests/golden/reproduced_rows.txt; a CPU test validates every stored witness again with validate.py (seconds), so
the expensive rows stay pinned without being solved again.  Allreduce rows are not searched: each is an
Allgather row composed with its inverse (section 3.5), which the composer's tests pin.
"""
from __future__ import annotations

import os
import sys
import time

import numpy as np

from . import collective as col
from . import synthesize as syn
from . import topology as tp
from .schedule import Schedule
from .validate import validate

GOLDEN = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "tests", "golden")
WITNESSES = os.path.join(GOLDEN, "witnesses")
MAKE = {"allgather": lambda P, C: col.allgather(P, C), "broadcast": lambda P, C: col.broadcast(P, C, 0),
        "gather": lambda P, C: col.gather(P, C, 0), "alltoall": lambda P, C: col.alltoall(P, C)}
TABLES = (("table5_z52.txt", "ring8", lambda: tp.ring(8)), ("table4_dgx1.txt", "dgx1", lambda: tp.dgx1()))


def rows(name):
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                coll, C, S, R, a, b, opt = line.split()
                yield coll, int(C), int(S), int(R), opt


def attempt(topo, coll, S, R, limit):
    """(verdict, seconds, schedule or None)"""
    t0 = time.time()
    try:
        s = syn.solve_instance(topo, coll, S, R, limit)
    except TimeoutError:
        return "timeout", time.time() - t0, None
    if s is None:
        return "infeasible", time.time() - t0, None
    ok = validate(topo, coll, s).ok
    return ("feasible" if ok else "INVALID"), time.time() - t0, (s if ok else None)


def witness_path(topo_name, name, C, S, R):
    return os.path.join(WITNESSES, f"{topo_name}_{name}_{C}_{S}_{R}.txt")


def write_witness(path, sched: Schedule):
    """rounds on the first line, then one send per line: chunk src dst step (every op is a copy)."""
    os.makedirs(os.path.dirname(path), exist_ok=True)
    with open(path, "w") as f:
        f.write("rounds " + " ".join(str(r) for r in sched.rounds) + "\n")
        for c, n, m, s, _ in sched.sends.tolist():
            f.write(f"{c} {n} {m} {s}\n")


def read_witness(path) -> Schedule:
    with open(path) as f:
        head = f.readline().split()
        assert head[0] == "rounds"
        sends = [[int(x) for x in line.split()] + [0] for line in f if line.strip()]
    return Schedule([int(r) for r in head[1:]], np.array(sends, dtype=np.int32).reshape(-1, 5))


def main():
    args = [a for a in sys.argv[1:] if a != "--write"]
    write = "--write" in sys.argv[1:]
    limit = float(args[0]) if args else 120.0
    report = []
    for table, topo_name, make_topo in TABLES:
        topo = make_topo()
        print(f"== {table} on {topo.name}")
        for name, C, S, R, opt in rows(table):
            if name == "allreduce":
                continue                                   # composed from the Allgather rows (section 3.5)
            coll = MAKE[name](8, C)
            res, dt, sched = attempt(topo, coll, S, R, limit)
            line = f"{name:10s} ({C},{S},{R}) {opt:10s} {res} in {dt:.1f} s"
            rec = [topo_name, name, C, S, R, opt, res, "-", "-"]
            if write and sched is not None:
                write_witness(witness_path(topo_name, name, C, S, R), sched)
            if opt in ("latency", "both") and S > 1:
                r2, d2, _ = attempt(topo, coll, S - 1, max(R, S - 1) + 8, limit)
                line += f"; with {S - 1} steps: {r2} ({d2:.1f} s)"
                rec[7] = r2
            if opt in ("bandwidth", "both") and R > S:
                r2, d2, _ = attempt(topo, coll, S, R - 1, limit)
                line += f"; with {R - 1} rounds: {r2} ({d2:.1f} s)"
                rec[8] = r2
            report.append(rec)
            print(line, flush=True)
    if write:
        with open(os.path.join(GOLDEN, "reproduced_rows.txt"), "w") as f:
            f.write("# Written by `python -m oracle.reproduce_tables --write` (exact search, oracle/synthesize.py): every\n"
                    "# non-Allreduce row of the paper's Tables 4 and 5, whether a schedule with that S and R exists (its\n"
                    "# witness is stored under witnesses/ and validated by a test), and, for rows the paper marks latency /\n"
                    "# bandwidth optimal, the verdict on the instance one step / one round cheaper.\n"
                    "# topology collective C S R optimality verdict one-step-fewer one-round-fewer\n")
            for rec in report:
                f.write(" ".join(str(x) for x in rec) + "\n")


if __name__ == "__main__":
    main()
