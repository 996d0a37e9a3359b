"""CPU oracle for IVFADC (TEST INFRASTRUCTURE ONLY): the paper's last experiment ("IVFADC with E-Tree": a coarse
quantiser of K' centroids, residual product quantisation, w probed inverted lists per query), written out from its
definition with numpy.  No kernel of the library implements this path yet; the oracle and its pins come first.

Conventions
  - A database vector x is stored as (cell, code): cell = its nearest coarse centroid, code = the product-quantiser
    encoding of the residual x - centroid[cell].  Its reconstruction is centroid[cell] + decode(code).
  - Decisions that pick an integer (the cell of a vector, the w probed cells of a query) are taken in float32 with
    the rule the library's encoder uses: a squared distance is the sum of its (a - b)^2 terms in dimension order, one
    rounding per operation, lowest index on ties.  Distances that are reported are float64.
  - A search returns, per query, the k smallest ||q - reconstruction||^2 over the vectors of its w probed cells,
    ascending by (distance, id); a query whose probed cells hold fewer than k vectors gets id -1 and +inf beyond.
"""
from __future__ import annotations

from typing import Optional, Tuple

import numpy as np

from . import decode, encode_f32


def sqdist_f32(x: np.ndarray, c: np.ndarray) -> np.ndarray:
    """[n][K'] float32 squared distances, each the sum of its terms in dimension order, every operation rounded once."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    c = np.ascontiguousarray(c, dtype=np.float32)
    acc = np.zeros((x.shape[0], c.shape[0]), dtype=np.float32)
    for j in range(x.shape[1]):
        t = x[:, j, None] - c[None, :, j]          # float32 subtraction
        acc = acc + t * t                           # float32 product, then float32 sum: two roundings, no fused form
    return acc


def coarse_assign(x: np.ndarray, centroids: np.ndarray) -> np.ndarray:
    """Cell of every vector: the nearest centroid in float32, lowest index on ties.  int32 [n]."""
    return np.argmin(sqdist_f32(x, centroids), axis=1).astype(np.int32)      # argmin returns the first minimum


def residuals(x: np.ndarray, centroids: np.ndarray, cells: np.ndarray) -> np.ndarray:
    """x - centroid[cell] in float32 (one rounding per component)."""
    return np.ascontiguousarray(x, dtype=np.float32) - np.ascontiguousarray(centroids, dtype=np.float32)[cells]


def build(x: np.ndarray, centroids: np.ndarray, codebooks: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """(cells int32 [n], codes uint8 [n][M]) of a database: coarse assignment, then the residuals' encodings."""
    cells = coarse_assign(x, centroids)
    return cells, encode_f32(residuals(x, centroids, cells), codebooks)


def reconstruct(centroids: np.ndarray, codebooks: np.ndarray, cells: np.ndarray, codes: np.ndarray) -> np.ndarray:
    """float64 [n][d]: centroid[cell] + decode(code)."""
    return np.asarray(centroids, dtype=np.float64)[cells] + np.asarray(decode(codes, codebooks), dtype=np.float64)


def probes(q: np.ndarray, centroids: np.ndarray, w: int) -> np.ndarray:
    """The w cells a query probes: nearest centroids in float32, ascending by (distance, index).  int32 [Q][w]."""
    d = sqdist_f32(q, centroids)
    order = np.lexsort((np.broadcast_to(np.arange(d.shape[1]), d.shape), d), axis=1)
    return order[:, :w].astype(np.int32)


def search(q: np.ndarray, centroids: np.ndarray, codebooks: np.ndarray, cells: np.ndarray, codes: np.ndarray, k: int,
           w: int, ids: Optional[np.ndarray] = None) -> Tuple[np.ndarray, np.ndarray]:
    """(ids int32 [Q][k], dist float64 [Q][k]) as described in the module's header."""
    q = np.ascontiguousarray(q, dtype=np.float32)
    n = len(cells)
    idv = np.arange(n, dtype=np.int64) if ids is None else np.asarray(ids, dtype=np.int64)
    xhat = reconstruct(centroids, codebooks, cells, codes)
    pr = probes(q, centroids, w)
    out_i = np.full((len(q), k), -1, dtype=np.int32)
    out_d = np.full((len(q), k), np.inf, dtype=np.float64)
    for j in range(len(q)):
        cand = np.flatnonzero(np.isin(cells, pr[j]))
        diff = xhat[cand] - q[j].astype(np.float64)
        dist = np.einsum("ij,ij->i", diff, diff)
        order = np.lexsort((idv[cand], dist))[:k]
        out_i[j, :len(order)] = idv[cand][order]
        out_d[j, :len(order)] = dist[order]
    return out_i, out_d


def split_terms(q: np.ndarray, centroids: np.ndarray, codebooks: np.ndarray, cells: np.ndarray, codes: np.ndarray):
    """The three terms a table-based evaluation would use, float64:
         ||q - c - r||^2  =  ||q - c||^2  +  (||r||^2 + 2 <c, r>)  -  2 <q, r>
       coarse [Q][K'] depends on (query, cell); vec [n] on the stored vector alone; cross [Q][n] = -2 <q, r> is a sum
       of M table entries that depend on the query alone (scalar-product tables of the residual codebooks)."""
    q = np.asarray(q, dtype=np.float64)
    c = np.asarray(centroids, dtype=np.float64)
    r = np.asarray(decode(codes, codebooks), dtype=np.float64)
    coarse = ((q[:, None, :] - c[None, :, :]) ** 2).sum(-1)
    vec = (r * r).sum(-1) + 2.0 * np.einsum("ij,ij->i", c[cells], r)
    cross = -2.0 * (q @ r.T)
    return coarse, vec, cross
