import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

GOLDEN = os.path.join(ROOT, "tests", "golden")


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


def read_table(name):
    """Rows of a golden table: (collective, C, S, R, a, Fraction b, optimality)."""
    from fractions import Fraction
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if not line:
                continue
            coll, C, S, R, a, b, opt = line.split()
            rows.append((coll, int(C), int(S), int(R), int(a), Fraction(b), opt))
    return rows


def read_examples():
    out = {}
    with open(os.path.join(GOLDEN, "worked_examples.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                k, *v = line.split()
                out[k] = v
    return out
