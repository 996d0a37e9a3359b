"""CPU oracle (TEST INFRASTRUCTURE ONLY).

Thin ctypes access to ``pq_adc_oracle.c`` (plain C, double accumulation) plus a
pure-Python pointer trie (``oracle.trie``) used to check tree statistics on tiny
inputs.  Nothing in the product package may import this module; only the tests,
``__graft_entry__.smoke`` and the benchmark's CPU-baseline leg do.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pq_adc_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (-O2, OpenMP over outer loops only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp",
                               "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        c_i64, c_int = ctypes.c_int64, ctypes.c_int
        P = ctypes.c_void_p
        lib.orc_num_threads.restype = c_int
        lib.orc_kmeans.argtypes = [P, c_i64, c_int, c_int, c_int, c_int, P, P, P]
        lib.orc_encode.argtypes = [P, c_i64, c_int, c_int, c_int, P, P]
        lib.orc_encode_f32.argtypes = [P, c_i64, c_int, c_int, c_int, P, P]
        lib.orc_decode.argtypes = [P, c_i64, c_int, c_int, c_int, P, P]
        lib.orc_brute.argtypes = [P, P, c_i64, c_int, P]
        lib.orc_lut.argtypes = [P, c_int, c_int, c_int, P, P]
        lib.orc_adc_flat.argtypes = [P, P, c_i64, c_int, c_int, P]
        lib.orc_topk.argtypes = [P, P, c_i64, c_int, P, P]
        lib.orc_adc_all.argtypes = [P, c_i64, c_int, c_int, c_int, P, P, c_i64, P]
        lib.orc_search.argtypes = [P, c_i64, c_int, c_int, c_int, P, P, P, c_i64, c_int, P, P]
        for f in ("orc_kmeans", "orc_encode", "orc_encode_f32", "orc_decode", "orc_brute", "orc_lut", "orc_adc_flat",
                  "orc_topk", "orc_adc_all", "orc_search"):
            getattr(lib, f).restype = c_int
        _lib = lib
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _check(rc: int, what: str):
    if rc != 0:
        raise ValueError("oracle %s failed with code %d" % (what, rc))


def num_threads() -> int:
    return int(_load().orc_num_threads())


def kmeans_init_rows(n: int, M: int, K: int, seed: int) -> np.ndarray:
    """The random draw of the k-means initialisation: for every group, the first
    K entries of a seeded permutation of the n training rows."""
    rng = np.random.Generator(np.random.PCG64([int(seed), 7]))
    rows = np.empty((M, K), dtype=np.int64)
    for m in range(M):
        rows[m] = rng.permutation(n)[:K] if n >= K else rng.integers(0, n, size=K)
    return rows


def kmeans(x, M: int, K: int, iters: int, init_rows: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Returns (codebooks float32 [M][K][d/M], objective float64 [M][iters])."""
    x = _f32(x)
    n, d = x.shape
    init_rows = np.ascontiguousarray(init_rows, dtype=np.int64)
    assert init_rows.shape == (M, K)
    cb = np.zeros((M, K, d // max(M, 1)), dtype=np.float32)
    obj = np.zeros((M, max(iters, 0)), dtype=np.float64)
    _check(_load().orc_kmeans(_p(x), n, d, M, K, iters, _p(init_rows), _p(cb), _p(obj)), "kmeans")
    return cb, obj


def encode(x, codebooks) -> np.ndarray:
    x = _f32(x)
    cb = _f32(codebooks)
    M, K, ds = cb.shape
    n, d = x.shape
    assert d == M * ds
    codes = np.zeros((n, M), dtype=np.uint8)
    _check(_load().orc_encode(_p(x), n, d, M, K, _p(cb), _p(codes)), "encode")
    return codes


def encode_f32(x, codebooks) -> np.ndarray:
    """The nearest-codeword assignment decided in float32 (sequential sums, one rounding per operation)."""
    x = _f32(x)
    cb = _f32(codebooks)
    M, K, ds = cb.shape
    n, d = x.shape
    assert d == M * ds
    codes = np.zeros((n, M), dtype=np.uint8)
    _check(_load().orc_encode_f32(_p(x), n, d, M, K, _p(cb), _p(codes)), "encode_f32")
    return codes


def decode(codes, codebooks) -> np.ndarray:
    cb = _f32(codebooks)
    M, K, ds = cb.shape
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    n = codes.shape[0]
    out = np.zeros((n, M * ds), dtype=np.float64)
    _check(_load().orc_decode(_p(codes), n, M * ds, M, K, _p(cb), _p(out)), "decode")
    return out


def brute(q, xhat) -> np.ndarray:
    q = _f32(q)
    xhat = np.ascontiguousarray(xhat, dtype=np.float64)
    n, d = xhat.shape
    out = np.zeros(n, dtype=np.float64)
    _check(_load().orc_brute(_p(q), _p(xhat), n, d, _p(out)), "brute")
    return out


def lut(q, codebooks) -> np.ndarray:
    q = _f32(q)
    cb = _f32(codebooks)
    M, K, ds = cb.shape
    out = np.zeros((M, K), dtype=np.float64)
    _check(_load().orc_lut(_p(q), M * ds, M, K, _p(cb), _p(out)), "lut")
    return out


def adc_flat(lut_mk, codes) -> np.ndarray:
    lut_mk = np.ascontiguousarray(lut_mk, dtype=np.float64)
    M, K = lut_mk.shape
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    N = codes.shape[0]
    out = np.zeros(N, dtype=np.float64)
    _check(_load().orc_adc_flat(_p(lut_mk), _p(codes), N, M, K, _p(out)), "adc_flat")
    return out


def topk(dist, k: int, ids=None) -> Tuple[np.ndarray, np.ndarray]:
    dist = np.ascontiguousarray(dist, dtype=np.float64)
    N = dist.shape[0]
    ids_a = None if ids is None else np.ascontiguousarray(ids, dtype=np.int32)
    oi = np.zeros(k, dtype=np.int32)
    od = np.zeros(k, dtype=np.float64)
    _check(_load().orc_topk(_p(dist), _p(ids_a), N, k, _p(oi), _p(od)), "topk")
    return oi, od


def adc_all(queries, codebooks, codes) -> np.ndarray:
    """dist[Q][N] float64 for every (query, encoding) pair."""
    queries = _f32(queries)
    cb = _f32(codebooks)
    M, K, ds = cb.shape
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    Q, N = queries.shape[0], codes.shape[0]
    out = np.zeros((Q, N), dtype=np.float64)
    _check(_load().orc_adc_all(_p(queries), Q, M * ds, M, K, _p(cb), _p(codes), N, _p(out)), "adc_all")
    return out


def search(queries, codebooks, codes, k: int, ids=None) -> Tuple[np.ndarray, np.ndarray]:
    """(ids int32 [Q][k], dist float64 [Q][k]), ascending by (distance, id)."""
    queries = _f32(queries)
    cb = _f32(codebooks)
    M, K, ds = cb.shape
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    Q, N = queries.shape[0], codes.shape[0]
    ids_a = None if ids is None else np.ascontiguousarray(ids, dtype=np.int32)
    oi = np.zeros((Q, k), dtype=np.int32)
    od = np.zeros((Q, k), dtype=np.float64)
    _check(_load().orc_search(_p(queries), Q, M * ds, M, K, _p(cb), _p(codes), _p(ids_a), N, k,
                              _p(oi), _p(od)), "search")
    return oi, od


# ---- scalar-product tables (the paper's remark that ADC tables may hold scalar products instead of distances):
# ---- the definition written out in float64 with numpy

def lut_ip(q, codebooks) -> np.ndarray:
    """lut[m][k] = <q restricted to group m, codeword k of group m>, float64."""
    q = np.asarray(_f32(q), dtype=np.float64)
    cb = np.asarray(_f32(codebooks), dtype=np.float64)
    M, K, ds = cb.shape
    out = np.zeros((M, K), dtype=np.float64)
    for m in range(M):
        out[m] = cb[m] @ q[m * ds:(m + 1) * ds]
    return out


def adc_all_ip(queries, codebooks, codes) -> np.ndarray:
    """ip[Q][N] float64: scalar product of every query with every reconstructed vector, as the sum of table entries."""
    queries = _f32(queries)
    return np.stack([adc_flat(lut_ip(q, codebooks), codes) for q in queries])


def search_ip(queries, codebooks, codes, k: int, ids=None) -> Tuple[np.ndarray, np.ndarray]:
    """(ids int32 [Q][k], ip float64 [Q][k]): the k largest scalar products, descending, ties by ascending id."""
    allp = adc_all_ip(queries, codebooks, codes)
    oi = np.zeros((allp.shape[0], k), dtype=np.int32)
    od = np.zeros((allp.shape[0], k), dtype=np.float64)
    for j in range(allp.shape[0]):
        oi[j], neg = topk(-allp[j], k, ids)
        od[j] = -neg
    return oi, od


def adc_all_term(q, codebooks, codes, term) -> np.ndarray:
    """Distances with a leaf payload (the paper's Experiments section stores an additive quantiser's extra term on the
    leaf): float64 [Q][N], the flat sum of table entries of vector n plus term[n]."""
    term = np.asarray(term, dtype=np.float64)
    d = adc_all(q, codebooks, codes)
    assert term.shape == (d.shape[1],)
    return d + term[None, :]


def search_term(q, codebooks, codes, term, k: int, ids: Optional[np.ndarray] = None) -> Tuple[np.ndarray, np.ndarray]:
    """(ids [Q][k], distances float64 [Q][k]): the k smallest (distance + term, id) per query, by a full sort."""
    d = adc_all_term(q, codebooks, codes, term)
    idv = np.arange(d.shape[1], dtype=np.int64) if ids is None else np.asarray(ids, dtype=np.int64)
    out_i = np.zeros((d.shape[0], k), dtype=np.int64)
    out_d = np.zeros((d.shape[0], k), dtype=np.float64)
    for j in range(d.shape[0]):
        order = np.lexsort((idv, d[j]))[:k]
        out_i[j], out_d[j] = idv[order], d[j][order]
    return out_i, out_d


def rotate(x: np.ndarray, R: np.ndarray) -> np.ndarray:
    """y = R x for every row of x ([n][d] float32, R [d][d] float32): the preprocessing step of Optimized Product
    Quantization (the paper's Related Work lists it among the quantisers whose codes the tree stores).  Every
    component is accumulated in float64 over the dimensions in ascending order, one rounded addition per dimension
    (the product of two float32 values is exact in float64), and rounded to float32 once at the end: a plain
    definition whose bits a float32 pipeline can reproduce.  Returns float32 [n][d]."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    R = np.ascontiguousarray(R, dtype=np.float32)
    n, d = x.shape
    assert R.shape == (d, d)
    acc = np.zeros((n, d), dtype=np.float64)
    Rt = R.T.astype(np.float64)                       # Rt[j] = column j of R: the factors of x[:, j]
    for j in range(d):
        acc = acc + x[:, j:j + 1].astype(np.float64) * Rt[j][None, :]
    return acc.astype(np.float32)
