"""Pins for the IVFADC oracle (oracle/ivfadc.py): a hand-worked example, brute force over reconstructed vectors, the
term split a table-based evaluation rests on.  No GPU, and no kernel implements this path yet."""
import json
import os

import numpy as np
from scipy.spatial.distance import cdist

import oracle
from oracle import ivfadc

GOLD = os.path.join(os.path.dirname(__file__), "golden", "worked_example.json")


def _problem(seed=0, n=600, d=12, kc=9, M=3, K=8, q=11):
    rng = np.random.default_rng(seed)
    x = rng.normal(size=(n, d)).astype(np.float32) * 2
    qs = rng.normal(size=(q, d)).astype(np.float32) * 2
    cent, _ = oracle.kmeans(x, 1, kc, 5, oracle.kmeans_init_rows(n, 1, kc, seed))
    cent = cent[0]
    cells = ivfadc.coarse_assign(x, cent)
    res = ivfadc.residuals(x, cent, cells)
    cb, _ = oracle.kmeans(res, M, K, 5, oracle.kmeans_init_rows(n, M, K, seed + 1))
    cells2, codes = ivfadc.build(x, cent, cb)
    assert np.array_equal(cells, cells2)
    return x, qs, cent, cb, cells, codes


def test_ivfadc_golden_worked_example():
    g = json.load(open(GOLD))["ivfadc"]
    cent = np.array(g["centroids"], dtype=np.float32)
    cb = np.array(g["codebooks"], dtype=np.float32)
    x = np.array(g["vectors"], dtype=np.float32)
    q = np.array([g["query"]], dtype=np.float32)
    cells, codes = ivfadc.build(x, cent, cb)
    assert cells.tolist() == g["cells"] and codes.tolist() == g["codes"]
    assert np.array_equal(ivfadc.reconstruct(cent, cb, cells, codes), np.array(g["reconstructions"]))
    assert ivfadc.sqdist_f32(q, cent)[0].tolist() == g["coarse_sqdist"]
    for w, key in ((1, "top3_one_probe"), (2, "top3_two_probes")):
        ids, dist = ivfadc.search(q, cent, cb, cells, codes, 3, w)
        assert ids[0].tolist() == g[key]["ids"]
        assert dist[0].tolist() == [float(v) for v in g[key]["dist"]]


def test_ivfadc_all_cells_probed_is_exhaustive_search_over_reconstructions():
    x, qs, cent, cb, cells, codes = _problem(seed=1)
    xhat = ivfadc.reconstruct(cent, cb, cells, codes)
    # every vector lies in the cell of its nearest centroid (another routine), its residual is what was encoded
    assert np.array_equal(cells, np.argmin(cdist(x.astype(np.float64), cent.astype(np.float64), "sqeuclidean"), axis=1))
    assert np.array_equal(codes, oracle.encode(x - cent[cells], cb))          # float64 assignment: no near-ties here
    ids = np.random.default_rng(2).permutation(5000)[: len(x)].astype(np.int32)
    oi, od = ivfadc.search(qs, cent, cb, cells, codes, 20, len(cent), ids)
    brute = cdist(qs.astype(np.float64), xhat, "sqeuclidean")
    for j in range(len(qs)):
        order = np.lexsort((ids, brute[j]))[:20]
        assert np.array_equal(oi[j], ids[order]) and np.allclose(od[j], brute[j][order], rtol=1e-12)


def test_ivfadc_probed_lists_and_short_lists():
    x, qs, cent, cb, cells, codes = _problem(seed=3)
    xhat = ivfadc.reconstruct(cent, cb, cells, codes)
    w = 3
    pr = ivfadc.probes(qs, cent, w)
    exact = cdist(qs.astype(np.float64), cent.astype(np.float64), "sqeuclidean")
    assert np.array_equal(pr, np.argsort(exact, axis=1, kind="stable")[:, :w])           # no near-ties in this data
    assert np.array_equal(ivfadc.probes(x, cent, 1)[:, 0], cells)                          # a vector's cell is its first probe
    oi, od = ivfadc.search(qs, cent, cb, cells, codes, 15, w)
    for j in range(len(qs)):
        inside = np.flatnonzero(np.isin(cells, pr[j]))
        dist = ((xhat[inside] - qs[j].astype(np.float64)) ** 2).sum(1)
        order = np.lexsort((inside, dist))[:15]
        assert np.array_equal(oi[j], inside[order]) and np.allclose(od[j], dist[order], rtol=1e-12)
        # nothing outside the probed cells is ever returned, however close
        assert np.all(np.isin(cells[oi[j]], pr[j]))
    # a list shorter than k: padded with id -1 and +inf
    few = np.flatnonzero(cells == np.bincount(cells).argmin())
    k = len(few) + 2
    target = cent[cells[few[0]]][None].astype(np.float32)
    oi, od = ivfadc.search(target, cent, cb, cells, codes, k, 1)
    assert sorted(oi[0][: len(few)].tolist()) == sorted(few.tolist())
    assert oi[0][len(few):].tolist() == [-1, -1] and np.all(np.isinf(od[0][len(few):]))


def test_ivfadc_distance_splits_into_query_cell_vector_and_table_terms():
    x, qs, cent, cb, cells, codes = _problem(seed=4)
    xhat = ivfadc.reconstruct(cent, cb, cells, codes)
    coarse, vec, cross = ivfadc.split_terms(qs, cent, cb, cells, codes)
    brute = cdist(qs.astype(np.float64), xhat, "sqeuclidean")
    assert np.allclose(coarse[:, cells] + vec[None, :] + cross, brute, rtol=0, atol=1e-9)
    # the cross term is a sum of M entries of scalar-product tables of the residual codebooks (query only)
    for j in range(len(qs)):
        lut = oracle.lut_ip(qs[j], cb)
        assert np.allclose(cross[j], -2.0 * oracle.adc_flat(lut, codes), rtol=0, atol=1e-10)
