"""Send/receive pair lists of the classic reduction trees the paper compares against (Section 4: binomial
tree, pipeline, binary tree), every segment through the same tree, for replay tests.  Test input only: no
times, no arithmetic of the method.  Within a segment every processor is listed after all it receives."""
from __future__ import annotations

import numpy as np


def _repeat(pairs, q):
    src = np.array([s for s, _ in pairs] * q, np.int32)
    dst = np.array([d for _, d in pairs] * q, np.int32)
    seg = np.repeat(np.arange(q, dtype=np.int32), len(pairs))
    return src, dst, seg


def pipeline(p: int, q: int):
    """A chain: processor i sends to i-1, the far end first."""
    return _repeat([(i, i - 1) for i in range(p - 1, 0, -1)], q)


def binomial(p: int, q: int):
    """Round r: every processor whose lowest set bit is 2^r sends to the one 2^r below it."""
    pairs, r = [], 0
    while (1 << r) < p:
        pairs += [(i, i - (1 << r)) for i in range(p) if i % (2 << r) == (1 << r)]
        r += 1
    return _repeat(pairs, q)


def binary(p: int, q: int):
    """Heap-shaped binary tree: the children of i are 2i+1 and 2i+2; deepest processors first."""
    return _repeat([(i, (i - 1) // 2) for i in range(p - 1, 0, -1)], q)
