"""Exhaustive search for the fewest steps on tiny graphs (oracle side; test infrastructure).

Used only to confirm, independently of the diameter and bandwidth bounds,
the minimal step counts of small rings and a few hand-made graphs, and that
the greedy generator reaches them there.  Non-combining collectives with
point-to-point constraints only.

The search is breadth first over whole states V_s (section 3.3's run), one
layer per step.  Within a step every directed link n -> n' with budget
b * r_s carries a subset of the chunks n holds and n' lacks.  Only maximal
subsets are tried: the run is monotone (V only grows and a larger V can
replay any continuation of a smaller one, dropping the sends whose chunk
already arrived), so sending fewer chunks on a link than it could carry never
reaches the post-condition sooner.  All maximal subsets ARE enumerated, and
all combinations over links, so the first layer that contains a state
covering post gives the true minimum.
"""
from __future__ import annotations

from itertools import combinations, product
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

from .collective import Collective
from .schedule import COPY, Schedule
from .topology import Topology


def _bit(c: int, n: int, P: int) -> int:
    return 1 << (c * P + n)


def _mask(rel: np.ndarray) -> int:
    G, P = rel.shape
    m = 0
    for c in range(G):
        for n in range(P):
            if rel[c, n]:
                m |= _bit(c, n, P)
    return m


def search(topo: Topology, coll: Collective, rounds: Sequence[int],
           state_limit: int = 200000) -> Optional[Schedule]:
    """A valid schedule with exactly the given rounds per step, or None if none exists."""
    if coll.combining:
        raise ValueError("search handles non-combining collectives")
    for L, b in topo.bw:
        if len(L) != 1:
            raise ValueError("search handles point-to-point constraints only")
    P, G = coll.num_nodes, coll.num_chunks
    cap = {next(iter(L)): b for L, b in topo.bw if b > 0}
    links = sorted(cap)
    start, goal = _mask(coll.pre), _mask(coll.post)
    layer: Dict[int, Tuple[Optional[int], Tuple]] = {start: (None, ())}
    history: List[Dict[int, Tuple[Optional[int], Tuple]]] = [layer]

    def unwind(state: int) -> Schedule:
        sends = []
        for s in range(len(history) - 1, 0, -1):
            prev, step_sends = history[s][state]
            sends = [(c, n, m, s - 1, COPY) for (c, n, m) in step_sends] + sends
            state = prev
        return Schedule(list(rounds[:len(history) - 1]), np.array(sends, dtype=np.int32).reshape(-1, 5))

    if start & goal == goal:
        return Schedule([], np.zeros((0, 5), dtype=np.int32))
    for s, r in enumerate(rounds):
        nxt: Dict[int, Tuple[Optional[int], Tuple]] = {}
        for state in layer:
            per_link = []
            for (n, m) in links:
                useful = [c for c in range(G) if state & _bit(c, n, P) and not state & _bit(c, m, P)]
                k = min(len(useful), cap[(n, m)] * r)
                per_link.append([tuple((c, n, m) for c in sub) for sub in combinations(useful, k)])
            for choice in product(*per_link):
                new = state
                flat = tuple(t for sub in choice for t in sub)
                for (c, n, m) in flat:
                    new |= _bit(c, m, P)
                if new not in nxt:
                    nxt[new] = (state, flat)
                    if len(nxt) > state_limit:
                        raise MemoryError("state limit reached; graph too large for the exhaustive search")
        history.append(nxt)
        layer = nxt
        for state in layer:
            if state & goal == goal:
                return _dedupe(unwind(state), coll)
    return None


def _dedupe(sched: Schedule, coll: Collective) -> Schedule:
    """Drop sends whose chunk reaches a node a second time in the same or a later step (keeps the first)."""
    have = coll.pre.astype(bool).copy()
    keep = []
    for s in range(sched.num_steps):
        got = set()
        for t in sched.sends.tolist():
            if t[3] != s:
                continue
            c, n, m = t[0], t[1], t[2]
            if have[c, m] or (c, m) in got:
                continue
            got.add((c, m))
            keep.append(t)
        for (c, m) in got:
            have[c, m] = True
    return Schedule(sched.rounds, np.array(keep, dtype=np.int32).reshape(-1, 5))


def min_steps(topo: Topology, coll: Collective, max_steps: int = 8, rounds_per_step: int = 1) -> Tuple[int, Schedule]:
    """Smallest S for which a schedule with r_s = rounds_per_step exists, with a witness."""
    for S in range(1, max_steps + 1):
        found = search(topo, coll, [rounds_per_step] * S)
        if found is not None:
            return S, found
    raise RuntimeError("no schedule within max_steps")
