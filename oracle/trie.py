"""Pointer-based encoding tree on tiny inputs (TEST INFRASTRUCTURE ONLY).

A deliberately naive prefix tree built by inserting encodings one by one
(section "Encoding Tree"): every node stands for one chunk of the encoding;
a node below which only one distinct encoding remains is a leaf that carries
the rest of that encoding as its postfix, and all vectors with that encoding
are associated with the leaf.  The walk follows the section "Distance
Computation with Hierarchical Memory Structure": depth-first, with a distance
context holding the partial sum of every level on the current path, so a shared
prefix is added once.

Used to check (a) that tree and forest traversals give the flat ADC sum for
every vector, and (b) node counts / postfix lengths / lookup counts that the
library's own builder reports.  Pure Python: keep inputs to a few thousand codes.
"""
from __future__ import annotations

from typing import Dict, List, Sequence

import numpy as np


class _Node:
    __slots__ = ("children", "ids", "count")

    def __init__(self):
        self.children: Dict[int, "_Node"] = {}
        self.ids: List[int] = []
        self.count = 0          # number of distinct encodings below (set by _finish)


class EncodingTree:
    """Tree over chunks [c0, c1) of the codes."""

    def __init__(self, codes: np.ndarray, c0: int = 0, c1: int | None = None):
        codes = np.asarray(codes)
        self.c0 = c0
        self.c1 = codes.shape[1] if c1 is None else c1
        self.D = self.c1 - self.c0
        self.N = codes.shape[0]
        self.root = _Node()
        for n in range(self.N):
            node = self.root
            for m in range(self.c0, self.c1):
                node = node.children.setdefault(int(codes[n, m]), _Node())
            node.ids.append(n)
        self._finish(self.root)

    def _finish(self, node: _Node) -> int:
        if not node.children:
            node.count = 1
        else:
            node.count = sum(self._finish(c) for c in node.children.values())
        return node.count

    def stats(self) -> dict:
        """Internal nodes per level, leaves per level, total postfix length, lookups.

        Levels are 1-based: a node at level l holds chunk c0+l-1.  A node (other
        than the root) below which more than one distinct encoding lies is
        internal; otherwise the first such node on a path is the leaf and the
        remaining D-l chunks are its postfix.
        """
        D = self.D
        nI = [0] * (D + 1)
        nL = [0] * (D + 1)
        sumP = 0
        stack = [(self.root, 0)]
        while stack:
            node, lev = stack.pop()
            for child in node.children.values():
                if child.count > 1:
                    nI[lev + 1] += 1
                    stack.append((child, lev + 1))
                else:
                    nL[lev + 1] += 1
                    sumP += D - (lev + 1)
        L1, L2 = sum(nI), sum(nL)
        return {
            "D": D, "N": self.N, "nI": nI[1:], "nL": nL[1:], "L1": L1, "L2": L2, "sumP": sumP,
            "lookups": L1 + L2 + sumP,                       # one per node plus one per postfix chunk
            "paper_bytes": 4 * self.N + 2 * (L1 + L2) + sumP,  # Hierarchical Memory Structure size
        }

    def distances(self, lut: np.ndarray) -> np.ndarray:
        """Per-vector partial distance over this tree's chunks, by depth-first walk.

        lut is the full [M][K] table of one query; level l uses row c0+l-1.
        """
        out = np.full(self.N, np.nan, dtype=np.float64)
        ctx = [0.0] * (self.D + 1)          # distance context: ctx[l] = partial sum down to level l

        def leaf_distance(node: _Node, lev: int, acc: float) -> None:
            # follow the single remaining path: the postfix
            while node.children:
                (code, child), = node.children.items()
                lev += 1
                acc += lut[self.c0 + lev - 1, code]
                node = child
            for i in node.ids:
                out[i] = acc

        def walk(node: _Node, lev: int) -> None:
            for code in sorted(node.children):
                child = node.children[code]
                part = ctx[lev] + lut[self.c0 + lev, code]
                if child.count > 1:
                    ctx[lev + 1] = part
                    walk(child, lev + 1)
                else:
                    leaf_distance(child, lev + 1, part)

        walk(self.root, 0)
        return out


def forest_distances(codes: np.ndarray, lut: np.ndarray, chunk_begin: Sequence[int]) -> np.ndarray:
    """Section "Encoding Forests": one tree per chunk group, per-tree result arrays
    indexed by vector id, summed element-wise in tree order."""
    total = np.zeros(codes.shape[0], dtype=np.float64)
    for t in range(len(chunk_begin) - 1):
        total += EncodingTree(codes, chunk_begin[t], chunk_begin[t + 1]).distances(lut)
    return total
