"""(alpha, beta) cost of a schedule (oracle side; test infrastructure).

Section 3.6 of the paper: with the L input bytes cut into C chunks, step s
with r_s rounds takes alpha + (r_s / C) * L * beta, so the whole algorithm
takes S * alpha + (R / C) * L * beta.  The pair (S, R/C) is the (latency
cost, bandwidth cost) by which section 3.7 orders algorithms.
"""
from __future__ import annotations

from fractions import Fraction
from typing import Sequence, Tuple


def cost_pair(C: int, S: int, R: int) -> Tuple[int, Fraction]:
    """(a, b) such that the running time is a*alpha + b*L*beta."""
    return S, Fraction(R, C)


def step_time(r_s: int, C: int, L: float, alpha: float, beta: float) -> float:
    return alpha + (r_s / C) * L * beta


def running_time(C: int, rounds: Sequence[int], L: float, alpha: float, beta: float) -> float:
    return sum(step_time(r, C, L, alpha, beta) for r in rounds)


def dominates(p: Tuple[int, Fraction], q: Tuple[int, Fraction]) -> bool:
    """p is at least as good as q in both costs and better in one (section 3.7's Pareto order)."""
    return p[0] <= q[0] and p[1] <= q[1] and p != q
