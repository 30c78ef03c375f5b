"""Validity of a candidate solution (oracle side; test infrastructure).

Section 3.3 of the paper: the run V_0 .. V_S of a schedule (Q, T) starts at
V_0 = pre and V_{s+1} = V_s + {(c, n') : (c, n) in V_s and (c, n, n', s) in T};
the schedule is valid if the post-condition is reached and, for every step s
and every constraint (L, b), the number of sends of step s on edges of L is at
most b * r_s.

Readings taken here:
  * The text prints "V_S subseteq post"; that is trivially true for Allgather
    and false for Gather, so it is read as post subseteq V_S (which is what
    constraint C2, time(c,n) <= S for (c,n) in post, says).
  * Steps are 0-based.
  * A send needs a usable link: (n, n') in E (section 3.4).

Combining collectives have no formal run in the paper, only the prose of
section 3.5 (a node receives the versions of a chunk and applies the
reduction).  The extension used here tracks, for every (c, n), the set K(c, n)
of ranks whose input is summed into the value stored there:
  * K_0(c, n) = {n} for (c, n) in pre.
  * COPY  n -> n': K(c, n') := K(c, n).
  * REDUCE n -> n': needs K(c, n) and K(c, n') disjoint (nothing is counted
    twice); K(c, n') := K(c, n') + K(c, n); afterwards (c, n) is *consumed*:
    reading it again is an error until a COPY overwrites it.
  * post: K_S(c, n) = all ranks for every (c, n) in post.
Within one step all reads see the state at the start of the step.  To make
that true without a snapshot, a step may not read and write the same (c, n),
and a COPY destination may be written by one send only and not reduced into
in the same step.
"""
from __future__ import annotations

import enum
from dataclasses import dataclass
from typing import Dict, List, Optional, Set, Tuple

import numpy as np

from .collective import Collective
from .schedule import CHUNK, COPY, DST, OP, REDUCE, SRC, STEP, Schedule
from .topology import Topology


class Verdict(enum.Enum):
    OK = "OK"
    INVALID_ARG = "INVALID_ARG"          # index out of range, bad rounds, unknown op, REDUCE in a non-combining collective
    SEND_NO_LINK = "SEND_NO_LINK"        # (n, n') not a usable link
    SEND_NO_SOURCE = "SEND_NO_SOURCE"    # (c, n) not in V_s / consumed
    BANDWIDTH = "BANDWIDTH"              # more than b * r_s sends over some constraint
    HAZARD = "HAZARD"                    # read+write of one (c, n) in a step, double write, double count
    POSTCONDITION = "POSTCONDITION"      # post not reached


@dataclass
class Report:
    verdict: Verdict
    detail: str = ""
    step: int = -1
    # filled when verdict is OK
    num_steps: int = 0
    num_rounds: int = 0
    k: int = 0
    links_used_per_step: Optional[List[int]] = None   # number of distinct directed links carrying a send

    @property
    def ok(self) -> bool:
        return self.verdict is Verdict.OK


def validate(topo: Topology, coll: Collective, sched: Schedule) -> Report:
    P, G = coll.num_nodes, coll.num_chunks
    S = sched.num_steps
    sends = sched.sends
    if topo.num_nodes != P:
        return Report(Verdict.INVALID_ARG, "topology and collective disagree on P")
    if S < 1 or any(r < 1 for r in sched.rounds):
        return Report(Verdict.INVALID_ARG, "every step needs at least one round")
    for i, (c, n, m, s, op) in enumerate(sends.tolist()):
        if not (0 <= c < G and 0 <= n < P and 0 <= m < P and 0 <= s < S) or n == m:
            return Report(Verdict.INVALID_ARG, f"send {i} out of range")
        if op not in (COPY, REDUCE):
            return Report(Verdict.INVALID_ARG, f"send {i}: unknown op")
        if op == REDUCE and not coll.combining:
            return Report(Verdict.INVALID_ARG, f"send {i}: REDUCE in a non-combining collective")

    links = set(topo.edges())
    for i, (c, n, m, s, op) in enumerate(sends.tolist()):
        if (n, m) not in links:
            return Report(Verdict.SEND_NO_LINK, f"send {i}: no link {n}->{m}", s)

    full = frozenset(range(P))
    # K[(c, n)] = contribution set, absent key = chunk not present / consumed
    K: Dict[Tuple[int, int], frozenset] = {}
    for c in range(G):
        for n in range(P):
            if coll.pre[c, n]:
                K[(c, n)] = frozenset([n]) if coll.combining else full
    links_used: List[int] = []

    for s in range(S):
        step_sends = [t for t in sends.tolist() if t[STEP] == s]
        # bandwidth: every constraint (L, b) admits at most b * r_s sends on its edges
        for L, b in topo.bw:
            cnt = sum(1 for t in step_sends if (t[SRC], t[DST]) in L)
            if cnt > b * sched.rounds[s]:
                return Report(Verdict.BANDWIDTH, f"step {s}: {cnt} sends over a constraint of {b} x {sched.rounds[s]}", s)
        # every source must hold the chunk at the start of the step
        for (c, n, m, _, op) in step_sends:
            if (c, n) not in K:
                return Report(Verdict.SEND_NO_SOURCE, f"step {s}: ({c},{n}) not present", s)
            if op == REDUCE and (c, m) not in K:
                return Report(Verdict.SEND_NO_SOURCE, f"step {s}: reduce into absent ({c},{m})", s)
        # hazards inside the step
        read: Set[Tuple[int, int]] = {(c, n) for (c, n, m, _, op) in step_sends}
        copy_dst: Set[Tuple[int, int]] = set()
        red_dst: Set[Tuple[int, int]] = set()
        for (c, n, m, _, op) in step_sends:
            if (c, m) in read:
                return Report(Verdict.HAZARD, f"step {s}: ({c},{m}) both read and written", s)
            if op == COPY:
                if (c, m) in copy_dst or (c, m) in red_dst:
                    return Report(Verdict.HAZARD, f"step {s}: ({c},{m}) written twice", s)
                copy_dst.add((c, m))
            else:
                if (c, m) in copy_dst:
                    return Report(Verdict.HAZARD, f"step {s}: ({c},{m}) copied and reduced into", s)
                red_dst.add((c, m))
        # apply the step on the start-of-step state
        newK = dict(K)
        consumed: Set[Tuple[int, int]] = set()
        for (c, n, m, _, op) in step_sends:
            if op == COPY:
                newK[(c, m)] = K[(c, n)]
            else:
                if newK[(c, m)] & K[(c, n)]:
                    return Report(Verdict.HAZARD, f"step {s}: rank counted twice in ({c},{m})", s)
                newK[(c, m)] = newK[(c, m)] | K[(c, n)]
                consumed.add((c, n))
        for key in consumed:
            del newK[key]
        K = newK
        links_used.append(len({(t[SRC], t[DST]) for t in step_sends}))

    for c in range(G):
        for n in range(P):
            if coll.post[c, n] and K.get((c, n)) != full:
                return Report(Verdict.POSTCONDITION, f"({c},{n}) not {'fully reduced' if coll.combining else 'present'} at the end")
    return Report(Verdict.OK, "", -1, S, sched.num_rounds, sched.k, links_used)


def run(coll: Collective, sched: Schedule) -> List[np.ndarray]:
    """The run V_0 .. V_S of section 3.3 for a non-combining schedule, as G x P 0/1 arrays."""
    V = coll.pre.astype(bool).copy()
    out = [V.copy()]
    for s in range(sched.num_steps):
        nxt = V.copy()
        for (c, n, m, st, op) in sched.sends.tolist():
            if st == s and V[c, n]:
                nxt[c, m] = True
        V = nxt
        out.append(V.copy())
    return out
