"""Exact synthesis of small schedules and the Pareto search of Algorithm 1 (oracle side; test infrastructure).

The paper decides an instance (G, S, R, P, B, pre, post) with an SMT solver over the encoding
C1-C6 of section 3.4.  Here the same question -- does a valid k-synchronous schedule with S
steps and R rounds exist -- is put to an exact integer-programming solver (HiGHS through
scipy.optimize.milp) over a time-indexed formulation of the definitions of section 3.3:

    x[c, e, s] in {0,1}   chunk c crosses link e = (n, n') during step s            (a send of T)
    h[c, n, s] in {0,1}   chunk c may be used at node n at the start of step s      (upper bound on V_s)
    r[s]       integer    rounds of step s, r[s] >= 1, sum r[s] = R                 (Q, constraint C6)

    h[c, n, 0] = pre(c, n)                                                         (C1)
    x[c, (n, n'), s] <= h[c, n, s]                         a send needs the chunk   (C4)
    h[c, n', s+1] <= h[c, n', s] + sum_n x[c, (n, n'), s]  the run V_{s+1}
    h[c, n, S] = 1 for (c, n) in post                                               (C2)
    sum_{s, n} x[c, (n, n'), s] <= 1 (= 0 on pre)          one receive per chunk    (C3)
    sum_{c, e in L} x[c, e, s] <= b * r[s]  for (L, b) in B                         (C5)

It is the "Boolean per tuple" encoding the paper found too slow for Z3 on its largest instance;
for the small rows of its tables an MILP solver handles it in seconds.  The answer is exact:
either a schedule (checked again by validate.py) or a proof that none exists.

pareto_frontier walks the Pareto frontier of (steps, bandwidth cost R/C) that Algorithm 1 reports:
per step count, from the diameter upwards, the cheapest feasible R/C among S <= R <= S + k, until the
bandwidth floor is met.  One reading: a point whose R/C is no better than one already found with
fewer steps is dominated (section 3.7's definition) and the paper's tables list none, so only
costs that improve on the best found so far are tried.
"""
from __future__ import annotations

from fractions import Fraction
from typing import Callable, Iterator, List, Optional, Sequence, Tuple

import numpy as np
from scipy.optimize import Bounds, LinearConstraint, milp
from scipy.sparse import coo_matrix

from .collective import Collective
from .schedule import COPY, Schedule
from .topology import Topology, allgather_bandwidth_bound, diameter


def solve_instance(topo: Topology, coll: Collective, S: int, R: int, time_limit: float = 120.0) -> Optional[Schedule]:
    """A valid schedule with exactly S steps and R rounds in total, or None when none exists.

    Raises TimeoutError when the solver gives up before deciding.
    """
    if coll.combining:
        raise ValueError("synthesis is for non-combining collectives; invert the result for combining ones")
    P, G = coll.num_nodes, coll.num_chunks
    if R < S:
        return None
    links = topo.edges()
    E = len(links)
    nx = G * E * S
    nh = G * P * (S + 1)
    nv = nx + nh + S

    def X(c, e, s):
        return (c * E + e) * S + s

    def H(c, n, s):
        return nx + (c * P + n) * (S + 1) + s

    def Rr(s):
        return nx + nh + s

    rows, cols, vals, lo, hi = [], [], [], [], []
    row = 0

    def add(entries, lb, ub):
        nonlocal row
        for j, v in entries:
            rows.append(row); cols.append(j); vals.append(v)
        lo.append(lb); hi.append(ub)
        row += 1

    lb = np.zeros(nv)
    ub = np.ones(nv)
    for s in range(S):
        lb[Rr(s)], ub[Rr(s)] = 1, R - (S - 1)
    for c in range(G):
        for n in range(P):
            v = 1.0 if coll.pre[c, n] else 0.0
            lb[H(c, n, 0)] = ub[H(c, n, 0)] = v
            if coll.post[c, n]:
                lb[H(c, n, S)] = 1.0
    into = {n: [e for e, (a, b) in enumerate(links) if b == n] for n in range(P)}
    for c in range(G):
        for e, (a, b) in enumerate(links):
            for s in range(S):
                add([(X(c, e, s), 1.0), (H(c, a, s), -1.0)], -np.inf, 0.0)
        for n in range(P):
            for s in range(S):
                add([(H(c, n, s + 1), 1.0), (H(c, n, s), -1.0)] + [(X(c, e, s), -1.0) for e in into[n]], -np.inf, 0.0)
            recv = [(X(c, e, s), 1.0) for e in into[n] for s in range(S)]
            if recv:
                add(recv, 0.0, 0.0 if coll.pre[c, n] else 1.0)
    for (L, b) in topo.bw:
        idx = [e for e, l in enumerate(links) if l in L]
        if not idx:
            continue
        for s in range(S):
            add([(X(c, e, s), 1.0) for c in range(G) for e in idx] + [(Rr(s), -float(b))], -np.inf, 0.0)
    add([(Rr(s), 1.0) for s in range(S)], float(R), float(R))

    A = coo_matrix((vals, (rows, cols)), shape=(row, nv)).tocsr()
    cost = np.zeros(nv)
    cost[:nx] = 1.0                                    # fewest sends: no useless traffic in the witness
    res = milp(cost, constraints=LinearConstraint(A, np.array(lo), np.array(hi)), integrality=np.ones(nv),
               bounds=Bounds(lb, ub), options={"time_limit": time_limit, "disp": False})
    if res.status == 2:                                # infeasible
        return None
    if res.x is None:                                  # neither a schedule nor a proof
        raise TimeoutError(f"solver stopped without an answer: {res.message}")
    x = np.rint(res.x).astype(np.int64)
    sends = []
    for s in range(S):
        for c in range(G):
            for e, (a, b) in enumerate(links):
                if x[X(c, e, s)]:
                    sends.append((c, a, b, s, COPY))
    rounds = [int(x[Rr(s)]) for s in range(S)]
    return _prune(Schedule(rounds, np.array(sends, dtype=np.int32).reshape(-1, 5)), coll)


def _prune(sched: Schedule, coll: Collective) -> Schedule:
    """Drop sends that do not serve the post-condition (a witness may carry harmless extra sends)."""
    sends = sched.sends.tolist()
    needed = {(c, n) for c in range(coll.num_chunks) for n in range(coll.num_nodes) if coll.post[c, n] and not coll.pre[c, n]}
    keep = []
    for t in sorted(sends, key=lambda t: -t[3]):       # latest first: a kept send makes its source needed
        c, n, m = t[0], t[1], t[2]
        if (c, m) in needed:
            keep.append(t)
            if not coll.pre[c, n]:
                needed.add((c, n))
    keep.sort(key=lambda t: (t[3], t[0], t[2]))
    return Schedule(sched.rounds, np.array(keep, dtype=np.int32).reshape(-1, 5))


def frontier_candidates(S: int, k: int, floor: Fraction, beaten: Optional[Fraction]) -> List[Tuple[Fraction, int, int]]:
    """The (R / C, R, C) a k-synchronous algorithm with S steps can have (S <= R <= S + k, R / C no lower than the
    bandwidth floor) that would improve on the lowest bandwidth cost known at fewer steps, cheapest first."""
    seen = {}
    for R in range(S, S + k + 1):
        C = 1
        while Fraction(R, C) >= floor:
            ratio = Fraction(R, C)
            if beaten is None or ratio < beaten:
                seen.setdefault(ratio, (ratio, R, C))              # the same cost with fewer rounds and chunks first
            C += 1
    return sorted(seen.values())


def pareto_frontier(k: int, topo: Topology, make_collective: Callable[[int], Collective],
                    bandwidth_bound: Optional[Fraction] = None, max_steps: int = 16,
                    time_limit: float = 120.0) -> Iterator[Tuple[int, int, int, Schedule]]:
    """The Pareto frontier of (steps S, bandwidth cost R / C) over k-synchronous schedules, one point per S, by
    increasing S -- what Algorithm 1 of the paper reports, and the rows its Tables 4 and 5 mark as the frontier.

    A point (S, R / C) is on the frontier when a schedule exists and none with at most S steps has a lower R / C.
    S starts at the latency floor (the diameter) and the walk ends at the first point that meets the bandwidth
    floor, which no later point can improve on.  make_collective(C) builds the instance for C chunks per node.
    """
    floor = bandwidth_bound if bandwidth_bound is not None else allgather_bandwidth_bound(topo)
    beaten: Optional[Fraction] = None                               # lowest R / C of the points yielded so far
    for S in range(diameter(topo), max_steps + 1):
        for ratio, R, C in frontier_candidates(S, k, floor, beaten):
            witness = solve_instance(topo, make_collective(C), S, R, time_limit)
            if witness is None:
                continue                                            # proved infeasible: try the next cheapest cost
            yield C, S, R, witness
            beaten = ratio
            break
        if beaten is not None and beaten == floor:
            return


def pareto_synthesize(k: int, topo: Topology, make_collective: Callable[[int], Collective],
                      bandwidth_bound: Optional[Fraction] = None, max_steps: int = 16,
                      time_limit: float = 120.0) -> List[Tuple[int, int, int, Schedule]]:
    """All frontier points as a list of (C, S, R, schedule): see pareto_frontier."""
    return list(pareto_frontier(k, topo, make_collective, bandwidth_bound, max_steps, time_limit))
