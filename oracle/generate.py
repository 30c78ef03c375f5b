"""Simple schedule generators (oracle side; test infrastructure).

The paper finds schedules with an SMT solver (section 3.4); that is not
rebuilt.  These generators are this repository's own and only their OUTPUTS
are trusted, through validate.py and the paper's lower bounds (diameter,
ingress bandwidth) and table rows.  What they borrow from the paper:

  * constraint C3 of section 3.4: a node receives a chunk at most once, so
    the sends of one chunk form a tree rooted at its owner;
  * constraint C4: a chunk is on the sender strictly before it is on the
    receiver;
  * section 3.5: a combining collective with one root per chunk is the
    inverse of a non-combining one on the reversed topology, and Allreduce is
    an Allgather preceded by its inverse.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

from .collective import Collective, allgather, allreduce, reducescatter
from .schedule import CHUNK, COPY, DST, OP, REDUCE, SRC, STEP, Schedule
from .topology import Topology


class GenerationError(RuntimeError):
    pass


def greedy_bfs(topo: Topology, coll: Collective, rounds: Optional[Sequence[int]] = None,
               max_steps: int = 1000) -> Schedule:
    """Greedy breadth-first schedule for a non-combining collective whose post is All (Allgather, Broadcast).

    Step by step: every constraint (L, b) gets a budget b * r_s.  A *need* is a
    pair (c, n') that lacks chunk c while some in-neighbour held it at the
    start of the step.  Needs are served in the order (fewest eligible
    sources, most nodes still lacking c, c, n'); the source chosen is the
    eligible in-neighbour whose link has the most budget left (lowest id on a
    tie).  A node receives each chunk once.  `rounds` gives r_s for the first
    steps; later steps get 1.
    """
    P, G = coll.num_nodes, coll.num_chunks
    if coll.combining or not coll.post.all():
        raise GenerationError("greedy_bfs handles non-combining collectives with post = All")
    links = topo.edges()
    in_nb: Dict[int, List[int]] = {n: [s for (s, d) in links if d == n] for n in range(P)}
    constraints_of: Dict[Tuple[int, int], List[int]] = {
        e: [i for i, (L, b) in enumerate(topo.bw) if e in L] for e in links}
    have = coll.pre.astype(bool).copy()
    sends: List[Tuple[int, int, int, int, int]] = []
    rounds_out: List[int] = []
    s = 0
    while not have.all():
        if s >= max_steps:
            raise GenerationError("step limit reached")
        r_s = int(rounds[s]) if rounds is not None and s < len(rounds) else 1
        budget = [b * r_s for (L, b) in topo.bw]

        def room(e):
            return min(budget[i] for i in constraints_of[e])

        lacking = (~have).sum(axis=1)           # per chunk: how many nodes still lack it
        needs = []
        for c in range(G):
            for n in range(P):
                if not have[c, n]:
                    elig = [m for m in in_nb[n] if have[c, m]]
                    if elig:
                        needs.append((len(elig), -int(lacking[c]), c, n, elig))
        needs.sort(key=lambda t: t[:4])
        got = []
        for (_, _, c, n, elig) in needs:
            best, best_room = -1, 0
            for m in elig:                       # ascending id, strict '>' keeps the lowest on ties
                rm = room((m, n))
                if rm > best_room:
                    best, best_room = m, rm
            if best < 0:
                continue
            for i in constraints_of[(best, n)]:
                budget[i] -= 1
            sends.append((c, best, n, s, COPY))
            got.append((c, n))
        if not got:
            raise GenerationError(f"step {s} could not send anything")
        for (c, n) in got:
            have[c, n] = True
        rounds_out.append(r_s)
        s += 1
    return Schedule(rounds_out, np.array(sends, dtype=np.int32))


def ring_allgather(P: int, C: int) -> Schedule:
    """Ring Allgather on the bidirectional P-ring: S = P-1 steps.

    Node n's i-th chunk is i*P + n (section 3.2.2).  Chunks with even i travel
    clockwise (n -> n+1), those with odd i counter-clockwise.  At step s node
    n forwards clockwise the clockwise chunks that originated at (n - s) mod P
    (and the mirror image the other way), the pipelined ring of section 2.4.
    Each directed link carries ceil(C/2) (or floor) chunks per step, so
    r_s = ceil(C/2) on a ring of 1 chunk/round links.
    """
    sends = []
    for s in range(P - 1):
        for n in range(P):
            for i in range(C):
                if i % 2 == 0:
                    origin = (n - s) % P
                    dst = (n + 1) % P
                else:
                    origin = (n + s) % P
                    dst = (n - 1) % P
                sends.append((i * P + origin, n, dst, s, COPY))
    r = (C + 1) // 2
    return Schedule([r] * (P - 1), np.array(sends, dtype=np.int32))


def invert(sched: Schedule, coll: Collective) -> Schedule:
    """Inverse of a non-combining schedule (section 3.5).

    Every send (c, n, n', s) becomes the REDUCE send (c, n', n, S-1-s) and Q is
    reversed.  The links used are those of the reversed topology.  Needs every
    (c, n) outside pre to be received exactly once (a tree per chunk, C3), so
    that each node forwards its partial sum exactly once, after it has
    received all its children's (C4 gives time(c, n) < time(c, n') for each
    send, which the inversion turns into "children first").

    The output is sorted by (step, destination, chunk, source): the order in
    which the versions arriving at one (chunk, destination) in one step are
    added is then fixed by the schedule alone.
    """
    S = sched.num_steps
    seen = set()
    for (c, n, m, s, op) in sched.sends.tolist():
        if op != COPY:
            raise GenerationError("only a non-combining schedule can be inverted")
        if coll.pre[c, m]:
            raise GenerationError(f"({c},{m}) is in pre but receives")
        if (c, m) in seen:
            raise GenerationError(f"({c},{m}) receives more than once")
        seen.add((c, m))
    inv = [(c, m, n, S - 1 - s, REDUCE) for (c, n, m, s, op) in sched.sends.tolist()]
    inv.sort(key=lambda t: (t[STEP], t[DST], t[CHUNK], t[SRC]))
    return Schedule(list(reversed(sched.rounds)), np.array(inv, dtype=np.int32).reshape(-1, 5))


def compose_allreduce(allgather_sched: Schedule, ag: Collective) -> Tuple[Schedule, Collective]:
    """Allreduce = inverse(Allgather) followed by the Allgather itself (section 3.5).

    Chunks per rank become G = P*C, steps 2S, rounds 2R, which is how every
    Allreduce row of the paper's tables relates to an Allgather row.
    """
    rs = invert(allgather_sched, ag)
    S = allgather_sched.num_steps
    shifted = allgather_sched.sends.copy()
    shifted[:, STEP] += S
    sends = np.concatenate([rs.sends, shifted], axis=0)
    return (Schedule(rs.rounds + allgather_sched.rounds, sends),
            allreduce(ag.num_nodes, ag.num_chunks))


def reducescatter_from(allgather_sched: Schedule, ag: Collective) -> Tuple[Schedule, Collective]:
    return invert(allgather_sched, ag), reducescatter(ag.num_nodes, ag.num_chunks)


def recursive_doubling_ring4() -> Schedule:
    """The 4-node example of section 3.1: neighbours (0,1), (2,3) swap their chunk, then (0,3), (1,2) swap both they hold.

    Two steps; the second moves two chunks per link, so Q = (1, 2) and R = 3.
    """
    sends = [(0, 0, 1, 0), (1, 1, 0, 0), (2, 2, 3, 0), (3, 3, 2, 0),
             (0, 0, 3, 1), (1, 0, 3, 1), (2, 3, 0, 1), (3, 3, 0, 1),
             (0, 1, 2, 1), (1, 1, 2, 1), (2, 2, 1, 1), (3, 2, 1, 1)]
    return Schedule([1, 2], np.array([list(t) + [COPY] for t in sends], dtype=np.int32))


def greedy_route(topo: Topology, coll: Collective, rounds: Optional[Sequence[int]] = None,
                 max_steps: int = 1000) -> Schedule:
    """Greedy shortest-path schedule for ANY non-combining collective (Gather, Scatter, Broadcast, Alltoall, ...).

    For every chunk a tree is fixed first: breadth-first from the nodes that hold it (pre) over the
    usable links; a node is *wanted* if it is in post or lies on the tree path to a node in post.  A
    wanted node's parent is, among its breadth-first predecessors, the one with the fewest children
    assigned so far over all chunks on that link (spreads an Alltoall over parallel shortest paths;
    lowest id on ties).  Every wanted node receives the chunk exactly once, from its parent (the
    one-receive rule C3 and the ordering rule C4 of section 3.4 hold by construction).

    Then the sends are packed into steps: in step s every constraint (L, b) has budget b * r_s; the
    pending sends whose parent already holds the chunk are served deepest-subtree-first (the longest
    remaining path below the receiver), ties by (chunk, receiver).
    """
    P, G = coll.num_nodes, coll.num_chunks
    if coll.combining:
        raise GenerationError("greedy_route handles non-combining collectives")
    links = topo.edges()
    in_nb: Dict[int, List[int]] = {n: [s for (s, d) in links if d == n] for n in range(P)}
    out_nb: Dict[int, List[int]] = {n: [d for (s, d) in links if s == n] for n in range(P)}
    constraints_of: Dict[Tuple[int, int], List[int]] = {
        e: [i for i, (L, b) in enumerate(topo.bw) if e in L] for e in links}
    link_load: Dict[Tuple[int, int], int] = {e: 0 for e in links}

    parent: Dict[Tuple[int, int], int] = {}          # (c, n) -> node it receives c from
    height: Dict[Tuple[int, int], int] = {}          # longest path of wanted nodes below (c, n)
    for c in range(G):
        holders = [n for n in range(P) if coll.pre[c, n]]
        targets = [n for n in range(P) if coll.post[c, n] and not coll.pre[c, n]]
        if not targets:
            continue
        if not holders:
            raise GenerationError(f"chunk {c} is nowhere in pre")
        dist = {n: 0 for n in holders}
        frontier = list(holders)
        while frontier:
            nxt = []
            for u in frontier:
                for v in out_nb[u]:
                    if v not in dist:
                        dist[v] = dist[u] + 1
                        nxt.append(v)
            frontier = nxt
        wanted = set()
        # farthest targets first, so that shared prefixes are reused by nearer ones
        for t in sorted(targets, key=lambda n: (-dist.get(n, -1), n)):
            if t not in dist:
                raise GenerationError(f"chunk {c} cannot reach node {t}")
            n = t
            while dist[n] > 0 and n not in wanted:
                wanted.add(n)
                preds = [m for m in in_nb[n] if dist.get(m, -1) == dist[n] - 1]
                # prefer a predecessor already on the tree, then the least loaded link
                best = min(preds, key=lambda m: (0 if (m in wanted or dist[m] == 0) else 1, link_load[(m, n)], m))
                parent[(c, n)] = best
                link_load[(best, n)] += 1
                n = best
        for n in sorted(wanted, key=lambda n: -dist[n]):
            height.setdefault((c, n), 0)
            p = parent[(c, n)]
            if dist[p] > 0:
                height[(c, p)] = max(height.get((c, p), 0), height[(c, n)] + 1)

    have = coll.pre.astype(bool).copy()
    pending = set(parent.keys())
    sends: List[Tuple[int, int, int, int, int]] = []
    rounds_out: List[int] = []
    s = 0
    while pending:
        if s >= max_steps:
            raise GenerationError("step limit reached")
        r_s = int(rounds[s]) if rounds is not None and s < len(rounds) else 1
        budget = [b * r_s for (L, b) in topo.bw]
        ready = sorted((key for key in pending if have[key[0], parent[key]]),
                       key=lambda key: (-height[key], key[0], key[1]))
        got = []
        for (c, n) in ready:
            e = (parent[(c, n)], n)
            if all(budget[i] > 0 for i in constraints_of[e]):
                for i in constraints_of[e]:
                    budget[i] -= 1
                sends.append((c, e[0], n, s, COPY))
                got.append((c, n))
        if not got:
            raise GenerationError(f"step {s} could not send anything")
        for key in got:
            have[key] = True
            pending.discard(key)
        rounds_out.append(r_s)
        s += 1
    if not rounds_out:
        rounds_out = [1]
    return Schedule(rounds_out, np.array(sends, dtype=np.int32).reshape(-1, 5))
