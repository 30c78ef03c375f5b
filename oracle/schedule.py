"""Candidate solution (Q, T) of section 3.3 (oracle side; test infrastructure).

Q = r_0 .. r_{S-1}, the rounds of each step (sum R); T a set of sends
(c, n, n', s): chunk c goes from node n to node n' during step s.  Steps are
numbered from 0 as in the definition of the run (the constraints C5/C6 of the
encoding count them from 1; a chunk "available at time t+1" was received
during step t).

Section 4 adds, for combining collectives, with which chunk a received chunk
is reduced: here each send carries an op, COPY (the destination's chunk is
replaced) or REDUCE (the source's version is added to the destination's).
The ORDER of the send array is part of the schedule: sends of one step that
reduce into the same (chunk, destination) are added in array order.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Sequence

import numpy as np

COPY = 0
REDUCE = 1

# column indices of the send array
CHUNK, SRC, DST, STEP, OP = range(5)


@dataclass
class Schedule:
    rounds: List[int]            # Q
    sends: np.ndarray            # (num_sends, 5) int32: chunk, src, dst, step, op

    def __post_init__(self):
        self.rounds = [int(r) for r in self.rounds]
        self.sends = np.asarray(self.sends, dtype=np.int32).reshape(-1, 5)

    @property
    def num_steps(self) -> int:      # S
        return len(self.rounds)

    @property
    def num_rounds(self) -> int:     # R
        return int(sum(self.rounds))

    @property
    def k(self) -> int:              # smallest k for which this is k-synchronous: R <= S + k (section 3.1)
        return self.num_rounds - self.num_steps

    def csr(self, chunks_per_node: int):
        """The (C, S, R) triple the paper's tables name an algorithm by."""
        return (chunks_per_node, self.num_steps, self.num_rounds)


def make_schedule(rounds: Sequence[int], sends: Sequence[Sequence[int]]) -> Schedule:
    arr = np.array([list(s) + [COPY] * (5 - len(s)) for s in sends], dtype=np.int32).reshape(-1, 5)
    return Schedule(list(rounds), arr)
