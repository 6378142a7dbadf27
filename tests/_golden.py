"""Readers of the small text fixtures under tests/golden/."""
import os

import numpy as np

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _lines(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return [l.strip() for l in f if l.strip() and not l.startswith("#")]


def flop_example():
    return {k: float(v) for k, v in (l.split() for l in _lines("paper_flop_example.txt"))}


def lp_ranks():
    return [(o, int(k), int(r)) for o, k, r in (l.split() for l in _lines("paper_lp_ranks.txt"))]


def walsh_rows():
    out = {}
    for l in _lines("walsh_rows.txt"):
        order, s, row = l.split()
        out[(int(order), int(s))] = np.array([1 if c == "+" else -1 for c in row], dtype=np.int64)
    return out


def selection_prefix_p8():
    out = {}
    for l in _lines("selection_prefix_p8.txt"):
        name, *pairs = l.split()
        out[name] = [tuple(int(t) for t in pr.split(",")) for pr in pairs]
    return out
