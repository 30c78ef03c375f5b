"""Re-derives the (C, S, R) rows of the paper's Tables 4 and 5 with the exact search (calls only oracle/ code).

Run from the repository root:  python -m oracle.reproduce_tables [seconds per instance]
For every row it reports whether a schedule with those S and R was found (and validated) and how long
the solver took; for rows marked latency / bandwidth optimal it also asks for the instance one step /
one round cheaper, which must be infeasible.  The largest rows may hit the time limit.
"""
from __future__ import annotations

import os
import sys
import time

from . import collective as col
from . import synthesize as syn
from . import topology as tp
from .validate import validate

GOLDEN = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "tests", "golden")
MAKE = {"allgather": lambda P, C: col.allgather(P, C), "broadcast": lambda P, C: col.broadcast(P, C, 0),
        "gather": lambda P, C: col.gather(P, C, 0), "alltoall": lambda P, C: col.alltoall(P, C)}


def rows(name):
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                coll, C, S, R, a, b, opt = line.split()
                yield coll, int(C), int(S), int(R), opt


def attempt(topo, coll, S, R, limit):
    t0 = time.time()
    try:
        s = syn.solve_instance(topo, coll, S, R, limit)
    except TimeoutError:
        return "timeout", time.time() - t0
    if s is None:
        return "infeasible", time.time() - t0
    return ("feasible" if validate(topo, coll, s).ok else "INVALID"), time.time() - t0


def main():
    limit = float(sys.argv[1]) if len(sys.argv) > 1 else 120.0
    for table, topo in (("table5_z52.txt", tp.ring(8)), ("table4_dgx1.txt", tp.dgx1())):
        print(f"== {table} on {topo.name}")
        for name, C, S, R, opt in rows(table):
            if name == "allreduce":
                continue                                   # composed from the Allgather rows (section 3.5)
            coll = MAKE[name](8, C)
            res, dt = attempt(topo, coll, S, R, limit)
            line = f"{name:10s} ({C},{S},{R}) {opt:10s} {res} in {dt:.1f} s"
            if opt in ("latency", "both") and S > 1:
                r2, d2 = attempt(topo, coll, S - 1, max(R, S - 1) + 8, limit)
                line += f"; with {S - 1} steps: {r2} ({d2:.1f} s)"
            if opt in ("bandwidth", "both") and R > S:
                r2, d2 = attempt(topo, coll, S, R - 1, limit)
                line += f"; with {R - 1} rounds: {r2} ({d2:.1f} s)"
            print(line, flush=True)


if __name__ == "__main__":
    main()
