"""Collectives as (pre, post) relations over (chunk, node) (oracle side; test infrastructure).

Table 1 of the paper gives four relations over [G] x [P]; Table 2 builds the
non-combining collectives from them.  Here [x] is read as {0, ..., x-1}: the
text prints {0, ..., x}, which would make "n = c mod P" range over P+1 nodes.

Section 3.2.2: node n's i-th input chunk has the global id i*P + n, so an
Allgather with C chunks per node has G = P*C global chunks and a Broadcast
has G = C.

Combining collectives (section 3.5) are written with the same two relations:
`pre` says where a *version* of the chunk lives at the start, `post` says
where the fully reduced chunk must be at the end.  Reducescatter is the
inverse of Allgather (pre All, post Scattered); Allreduce is pre All, post All.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np


def rel_all(G: int, P: int) -> np.ndarray:
    return np.ones((G, P), dtype=np.uint8)


def rel_root(G: int, P: int, root: int) -> np.ndarray:
    r = np.zeros((G, P), dtype=np.uint8)
    r[:, root] = 1
    return r


def rel_scattered(G: int, P: int) -> np.ndarray:
    r = np.zeros((G, P), dtype=np.uint8)
    for c in range(G):
        r[c, c % P] = 1
    return r


def rel_transpose(G: int, P: int) -> np.ndarray:
    r = np.zeros((G, P), dtype=np.uint8)
    for c in range(G):
        r[c, (c // P) % P] = 1
    return r


@dataclass(frozen=True)
class Collective:
    name: str
    num_nodes: int           # P
    num_chunks: int          # G, global
    pre: np.ndarray          # G x P, 0/1
    post: np.ndarray         # G x P, 0/1
    combining: bool = False
    chunks_per_node: Optional[int] = None   # C in the paper's evaluation tables

    def __post_init__(self):
        assert self.pre.shape == (self.num_chunks, self.num_nodes)
        assert self.post.shape == (self.num_chunks, self.num_nodes)


def to_global(name: str, C: int, P: int) -> int:
    """ToGlobal of Algorithm 1: global chunk count from the per-node count (section 3.2.2)."""
    if name in ("allgather", "gather"):
        return P * C
    if name in ("broadcast", "scatter"):
        return C
    if name in ("reducescatter", "allreduce", "reduce"):
        # every node starts with a version of EVERY chunk, so the per-node
        # count already is the global one (the tables' footnote: multiply the
        # Allgather row's C by P to get the Reducescatter's)
        return C
    if name == "alltoall":
        return P * C       # C counts chunks per node; a useful Alltoall needs C a multiple of P
    raise ValueError(name)


def allgather(P: int, C: int = 1) -> Collective:
    G = to_global("allgather", C, P)
    return Collective("allgather", P, G, rel_scattered(G, P), rel_all(G, P), False, C)


def gather(P: int, C: int = 1, root: int = 0) -> Collective:
    G = to_global("gather", C, P)
    return Collective("gather", P, G, rel_scattered(G, P), rel_root(G, P, root), False, C)


def alltoall(P: int, C: int) -> Collective:
    G = to_global("alltoall", C, P)
    return Collective("alltoall", P, G, rel_scattered(G, P), rel_transpose(G, P), False, C)


def broadcast(P: int, C: int = 1, root: int = 0) -> Collective:
    G = to_global("broadcast", C, P)
    return Collective("broadcast", P, G, rel_root(G, P, root), rel_all(G, P), False, C)


def scatter(P: int, C: int = 1, root: int = 0) -> Collective:
    G = to_global("scatter", C, P)
    return Collective("scatter", P, G, rel_root(G, P, root), rel_scattered(G, P), False, C)


def reducescatter(P: int, G: int) -> Collective:
    """Inverse of Allgather (section 3.5): every node starts with its own version of every chunk."""
    return Collective("reducescatter", P, G, rel_all(G, P), rel_scattered(G, P), True, G)


def reduce(P: int, C: int = 1, root: int = 0) -> Collective:
    """Inverse of Broadcast (section 3.5)."""
    G = to_global("reduce", C, P)
    return Collective("reduce", P, G, rel_all(G, P), rel_root(G, P, root), True, G)


def allreduce(P: int, G: int) -> Collective:
    """Reducescatter followed by Allgather (section 3.5); the tables count its chunks per node, so C = G."""
    return Collective("allreduce", P, G, rel_all(G, P), rel_all(G, P), True, G)


def compact_slots(coll: Collective, sends: np.ndarray):
    """A slot map that gives every rank room only for the chunks it ever holds.

    The paper numbers chunks globally (section 3.2.2) and leaves the placement inside a node's
    memory open.  Rank n gets one slot per chunk that is in pre at n or that some send delivers to
    n, in ascending chunk order; all ranks' buffers are sized to the largest count.  Returns
    (slot, slots_per_rank) with slot a G x P int32 array, -1 where rank n never holds chunk c.
    """
    G, P = coll.num_chunks, coll.num_nodes
    held = coll.pre.astype(bool).copy()
    for (c, n, m, s, op) in np.asarray(sends).reshape(-1, 5).tolist():
        held[c, m] = True
    slot = np.full((G, P), -1, dtype=np.int32)
    for n in range(P):
        k = 0
        for c in range(G):
            if held[c, n]:
                slot[c, n] = k
                k += 1
    return slot, int(held.sum(axis=0).max())
