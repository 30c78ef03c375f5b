"""Reader of the text schedule files under schedules/ (plain data in, binding descriptions out).

A schedule file carries everything sccl_plan_create needs except the element
type and count: the bandwidth relation B, the collective's pre/post relations
and the schedule (Q, T).  The files shipped here were written by
oracle/write_schedules.py; a synthesizer's output can be stored the same way.

Format, one record per line, '#' starts a comment:
    sccl-schedule 1
    name <text>
    collective <name> combining <0|1>
    nodes <P>
    chunks <G>
    chunks_per_node <C>
    pre  <all | scattered | transpose | root:<n> | rows>      (rows: G lines of P 0/1 digits follow)
    post <...>
    bw <b> <src>><dst> [<src>><dst> ...]                      one (L, b) per line
    slots <K>                                                 optional layout: G lines of P integers follow, the chunk
                                                              position of chunk c in rank n's buffer of K chunks, -1 = never held
    rounds <r_0> ... <r_{S-1}>
    sends <count>
    <chunk> <src> <dst> <step> <op>                           count lines, order significant
"""
from __future__ import annotations

import os
from dataclasses import dataclass
from typing import List, Optional, Tuple

import numpy as np

from . import sccl

SCHEDULE_DIR = os.path.join(os.path.dirname(os.path.abspath(__file__)), "schedules")


@dataclass
class ScheduleFile:
    name: str
    collective: str
    combining: bool
    num_nodes: int
    num_chunks: int
    chunks_per_node: int
    pre: np.ndarray
    post: np.ndarray
    bw: List[Tuple[List[Tuple[int, int]], int]]
    rounds: List[int]
    sends: np.ndarray
    slot: Optional[np.ndarray] = None        # G x P chunk positions, or None: chunk c at position c
    slots_per_rank: int = 0

    @property
    def positions_per_rank(self) -> int:
        """Chunks a rank buffer has room for."""
        return self.slots_per_rank if self.slot is not None else self.num_chunks

    def descriptions(self, dtype: str, elems_per_chunk: int):
        """(Topology, Collective, Schedule) for sccl_plan_create."""
        return (sccl.Topology(self.num_nodes, self.bw),
                sccl.Collective(self.num_chunks, self.pre, self.post, self.combining, dtype, elems_per_chunk,
                                self.slot, self.slots_per_rank),
                sccl.Schedule(self.rounds, self.sends))


def _relation(word: str, G: int, P: int, lines) -> np.ndarray:
    r = np.zeros((G, P), dtype=np.uint8)
    if word == "all":
        r[:] = 1
    elif word == "scattered":
        for c in range(G):
            r[c, c % P] = 1
    elif word == "transpose":
        for c in range(G):
            r[c, (c // P) % P] = 1
    elif word.startswith("root:"):
        r[:, int(word[5:])] = 1
    elif word == "rows":
        for c in range(G):
            row = next(lines)
            r[c] = [int(ch) for ch in row.strip()]
    else:
        raise ValueError(f"unknown relation {word}")
    return r


def load(path_or_name: str) -> ScheduleFile:
    path = path_or_name
    if not os.path.exists(path):
        path = os.path.join(SCHEDULE_DIR, path_or_name + ("" if path_or_name.endswith(".txt") else ".txt"))
    with open(path) as f:
        raw = [ln.split("#")[0].strip() for ln in f]
    lines = iter([ln for ln in raw if ln])
    head = next(lines).split()
    if head != ["sccl-schedule", "1"]:
        raise ValueError("not a schedule file")
    name = collective = ""
    combining = False
    P = G = C = 0
    pre = post = None
    bw: List[Tuple[List[Tuple[int, int]], int]] = []
    rounds: List[int] = []
    sends = np.zeros((0, 5), dtype=np.int32)
    slot, slots_per_rank = None, 0
    for ln in lines:
        w = ln.split()
        if w[0] == "name":
            name = " ".join(w[1:])
        elif w[0] == "collective":
            collective, combining = w[1], bool(int(w[3]))
        elif w[0] == "nodes":
            P = int(w[1])
        elif w[0] == "chunks":
            G = int(w[1])
        elif w[0] == "chunks_per_node":
            C = int(w[1])
        elif w[0] == "pre":
            pre = _relation(w[1], G, P, lines)
        elif w[0] == "post":
            post = _relation(w[1], G, P, lines)
        elif w[0] == "bw":
            edges = [tuple(int(x) for x in e.split(">")) for e in w[2:]]
            bw.append((edges, int(w[1])))
        elif w[0] == "slots":
            slots_per_rank = int(w[1])
            slot = np.array([[int(x) for x in next(lines).split()] for _ in range(G)], dtype=np.int32).reshape(G, P)
        elif w[0] == "rounds":
            rounds = [int(x) for x in w[1:]]
        elif w[0] == "sends":
            n = int(w[1])
            sends = np.array([[int(x) for x in next(lines).split()] for _ in range(n)], dtype=np.int32).reshape(-1, 5)
        else:
            raise ValueError(f"unknown record {w[0]}")
    return ScheduleFile(name, collective, combining, P, G, C, pre, post, bw, rounds, sends, slot, slots_per_rank)
