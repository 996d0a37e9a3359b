"""Pins for the CPU oracle: things the paper and the mathematics fix, none of
which is the oracle's own formula retyped.  Runs without a GPU."""
import json
import os

import numpy as np
import pytest
from scipy.spatial.distance import cdist

import oracle
from oracle.trie import EncodingTree, forest_distances
from workload import GaussianMixture

GOLD = os.path.join(os.path.dirname(__file__), "golden", "worked_example.json")


def _tiny(seed=0, n=64, d=8, M=4, K=4, q=5):
    rng = np.random.default_rng(seed)
    x = rng.normal(size=(n, d)).astype(np.float32)
    qs = rng.normal(size=(q, d)).astype(np.float32)
    cb, _ = oracle.kmeans(x, M, K, 5, oracle.kmeans_init_rows(n, M, K, seed))
    codes = oracle.encode(x, cb)
    return x, qs, cb, codes


# ---------------------------------------------------------------- hand-worked example
def test_golden_worked_example():
    g = json.load(open(GOLD))
    cb = np.array(g["codebooks"], dtype=np.float32)
    q = np.array(g["query"], dtype=np.float32)
    codes = np.array(g["codes"], dtype=np.uint8)
    lut = oracle.lut(q, cb)
    assert np.array_equal(lut, np.array(g["lut"]))
    dist = oracle.adc_flat(lut, codes)
    assert np.array_equal(dist, np.array(g["distances"]))
    ids, dd = oracle.topk(dist, 3)
    assert ids.tolist() == g["top3_ids"] and dd.tolist() == g["top3_dist"]
    sid, sdd = oracle.search(q[None], cb, codes, 3)
    assert sid[0].tolist() == g["top3_ids"] and sdd[0].tolist() == g["top3_dist"]
    enc = oracle.encode(np.array(g["encode_inputs"], dtype=np.float32), cb)
    assert enc.tolist() == g["encode_codes"]
    assert oracle.decode(np.array([[1, 0]], dtype=np.uint8), cb)[0].tolist() == g["decode_of_1_0"]
    allp = oracle.adc_all(q[None], cb, codes)
    assert np.array_equal(allp[0], np.array(g["distances"]))


def test_golden_kmeans_on_the_line():
    g = json.load(open(GOLD))["kmeans_1d"]
    x = np.array(g["x"], dtype=np.float32)
    cb, obj = oracle.kmeans(x, 1, 2, 3, np.array(g["init_rows"], dtype=np.int64))
    assert np.allclose(obj[0], g["objective"], rtol=1e-14)
    assert np.array_equal(cb, np.array(g["codebook"], dtype=np.float32))


def test_golden_tree_counts():
    g = json.load(open(GOLD))
    st = EncodingTree(np.array(g["codes"], dtype=np.uint8)).stats()
    for key, val in g["tree"].items():
        assert st[key] == val, key


# ---------------------------------------------------------------- ADC == distance to the decoded vector
@pytest.mark.parametrize("seed,d,M,K", [(0, 8, 4, 4), (1, 8, 2, 3), (2, 6, 1, 4), (3, 12, 3, 1), (4, 8, 8, 2)])
def test_adc_equals_bruteforce_on_decoded(seed, d, M, K):
    x, qs, cb, codes = _tiny(seed, 64, d, M, K)
    xhat = oracle.decode(codes, cb)
    for q in qs:
        adc = oracle.adc_flat(oracle.lut(q, cb), codes)
        ref = oracle.brute(q, xhat)
        assert np.allclose(adc, ref, rtol=1e-13, atol=1e-13)
        # library routine on the same decoded vectors (not the oracle's loop)
        lib = cdist(q[None].astype(np.float64), xhat, "sqeuclidean")[0]
        assert np.allclose(adc, lib, rtol=1e-12, atol=1e-12)


def test_adc_group_order_matters_transposition_detected():
    # codebooks that differ strongly between groups: swapping groups or
    # transposing the table would change the answer
    rng = np.random.default_rng(5)
    cb = rng.normal(size=(2, 3, 2)).astype(np.float32) * np.array([1.0, 10.0], dtype=np.float32)[:, None, None]
    codes = np.array([[0, 1], [1, 0], [2, 2], [0, 2]], dtype=np.uint8)
    q = rng.normal(size=4).astype(np.float32)
    xhat = np.concatenate([cb[0][codes[:, 0]], cb[1][codes[:, 1]]], axis=1).astype(np.float64)
    ref = ((q[None].astype(np.float64) - xhat) ** 2).sum(1)
    assert np.allclose(oracle.adc_flat(oracle.lut(q, cb), codes), ref, rtol=1e-13)
    assert np.array_equal(oracle.decode(codes, cb), xhat)


# ---------------------------------------------------------------- encoding picks the nearest codeword
def test_encode_is_optimal_by_exhaustive_search():
    x, _, cb, codes = _tiny(7, 200, 12, 3, 5)
    M, K, ds = cb.shape
    for m in range(M):
        dm = cdist(x[:, m * ds:(m + 1) * ds].astype(np.float64), cb[m].astype(np.float64), "sqeuclidean")
        chosen = dm[np.arange(len(x)), codes[:, m]]
        assert np.all(chosen <= dm.min(axis=1) + 1e-12)
        # lowest index among exact minima
        assert np.array_equal(codes[:, m], dm.argmin(axis=1))


# ---------------------------------------------------------------- k-means
def test_kmeans_objective_monotone():
    gm = GaussianMixture(16, 8, 1.1, (0.2, 1.0), (-4, 4), seed=3)
    x = gm.sample(2000, 11)
    cb, obj = oracle.kmeans(x, 4, 16, 8, oracle.kmeans_init_rows(2000, 4, 16, 1))
    assert np.all(np.diff(obj, axis=1) <= 1e-12)
    # the reported objective is the quantisation error of the centroids the iteration started from;
    # after the last update the error can only be lower still
    codes = oracle.encode(x, cb)
    err = ((x.astype(np.float64) - oracle.decode(codes, cb)) ** 2).reshape(2000, 4, 4).sum(2).mean(0)
    assert np.all(err <= obj[:, -1] + 1e-6)


def test_lossless_quantiser_gives_exact_distances():
    # at most K distinct sub-vectors per group and an initialisation that covers them:
    # the quantiser is lossless, so ADC must equal the exact squared distance
    rng = np.random.default_rng(9)
    M, K, ds = 3, 4, 2
    protos = rng.normal(size=(M, K, ds)).astype(np.float32)
    pick = rng.integers(0, K, size=(50, M))
    pick[:K] = np.arange(K)[:, None]           # every prototype occurs, rows 0..K-1
    x = np.concatenate([protos[m][pick[:, m]] for m in range(M)], axis=1)
    init = np.tile(np.arange(K, dtype=np.int64), (M, 1))
    cb, obj = oracle.kmeans(x, M, K, 4, init)
    assert np.all(obj == 0.0)
    codes = oracle.encode(x, cb)
    qs = rng.normal(size=(6, M * ds)).astype(np.float32)
    got = oracle.adc_all(qs, cb, codes)
    ref = cdist(qs.astype(np.float64), x.astype(np.float64), "sqeuclidean")
    assert np.allclose(got, ref, rtol=1e-12, atol=1e-12)


# ---------------------------------------------------------------- special cases
def test_M1_is_plain_vector_quantisation():
    x, qs, cb, codes = _tiny(11, 40, 6, 1, 4)
    for q in qs:
        ref = ((q.astype(np.float64)[None] - cb[0][codes[:, 0]].astype(np.float64)) ** 2).sum(1)
        assert np.allclose(oracle.adc_flat(oracle.lut(q, cb), codes), ref, rtol=1e-13)


def test_K1_all_distances_equal():
    x, qs, cb, codes = _tiny(12, 30, 8, 4, 1)
    assert np.all(codes == 0)
    d = oracle.adc_all(qs, cb, codes)
    assert np.all(d == d[:, :1])


def test_query_equal_to_reconstruction_has_zero_distance():
    x, _, cb, codes = _tiny(13, 30, 8, 4, 4)
    xhat = oracle.decode(codes, cb)
    n = 7
    q = xhat[n].astype(np.float32)           # codebooks are float32, so this is exact
    lut = oracle.lut(q, cb)
    assert all(lut[m, codes[n, m]] == 0.0 for m in range(4))
    assert oracle.adc_flat(lut, codes)[n] == 0.0
    assert np.all(lut >= 0.0)


# ---------------------------------------------------------------- top-k
def test_topk_is_prefix_of_lexicographic_sort():
    rng = np.random.default_rng(21)
    dist = rng.integers(0, 20, size=500).astype(np.float64)      # many exact ties
    ids = rng.permutation(500).astype(np.int32)
    order = np.lexsort((ids, dist))                               # library routine: by dist, then id
    for k in (1, 7, 100, 500):
        oi, od = oracle.topk(dist, k, ids)
        assert np.array_equal(oi, ids[order[:k]])
        assert np.array_equal(od, dist[order[:k]])
    oi, _ = oracle.topk(dist, 500, ids)
    assert sorted(oi.tolist()) == list(range(500))
    oi, od = oracle.topk(dist, 1)
    assert od[0] == dist.min() and oi[0] == int(np.flatnonzero(dist == dist.min())[0])


def test_search_matches_stepwise_calls():
    x, qs, cb, codes = _tiny(31, 300, 8, 4, 4)
    ids = (np.arange(300, dtype=np.int32) * 3 + 5)
    si, sd = oracle.search(qs, cb, codes, 10, ids)
    xhat = oracle.decode(codes, cb)
    for j, q in enumerate(qs):
        ref = cdist(q[None].astype(np.float64), xhat, "sqeuclidean")[0]
        order = np.lexsort((ids, oracle.adc_flat(oracle.lut(q, cb), codes)))[:10]
        assert np.array_equal(si[j], ids[order])
        assert np.allclose(sd[j], ref[order], rtol=1e-12)


# ---------------------------------------------------------------- tree / forest semantics and counts
@pytest.mark.parametrize("seed,M,K,n", [(0, 4, 3, 200), (1, 6, 2, 300), (2, 8, 4, 500), (3, 3, 5, 50)])
def test_tree_and_forest_walks_equal_flat(seed, M, K, n):
    rng = np.random.default_rng(seed)
    codes = rng.integers(0, K, size=(n, M)).astype(np.uint8)
    lut = rng.random(size=(M, K)) * 10
    flat = oracle.adc_flat(lut, codes)
    tree = EncodingTree(codes).distances(lut)
    assert np.allclose(tree, flat, rtol=1e-14)
    splits = [[0, M], [0, M // 2, M], list(range(M + 1))]
    for cb in splits:
        assert np.allclose(forest_distances(codes, lut, cb), flat, rtol=1e-13)


def test_tree_counts_closed_forms():
    D = 5
    # all encodings equal: one leaf at level 1 with postfix D-1
    st = EncodingTree(np.full((9, D), 3, dtype=np.uint8)).stats()
    assert (st["L1"], st["L2"], st["sumP"], st["nL"][0]) == (0, 1, D - 1, 1)
    assert st["lookups"] == D and st["paper_bytes"] == 4 * 9 + 2 * 1 + (D - 1)
    # all first chunks distinct: every encoding is a level-1 leaf; as many lookups as flat ADC
    rng = np.random.default_rng(0)
    c = rng.integers(0, 7, size=(6, D)).astype(np.uint8)
    c[:, 0] = np.arange(6)
    st = EncodingTree(c).stats()
    assert (st["L1"], st["L2"], st["sumP"]) == (0, 6, 6 * (D - 1)) and st["lookups"] == 6 * D
    # full enumeration of K**D encodings: K**l internal nodes at level l<D, all leaves at level D
    K, D = 3, 4
    grid = np.array(np.meshgrid(*[np.arange(K)] * D, indexing="ij")).reshape(D, -1).T.astype(np.uint8)
    st = EncodingTree(grid).stats()
    assert st["nI"] == [K, K * K, K ** 3, 0] and st["nL"] == [0, 0, 0, K ** 4] and st["sumP"] == 0
    assert st["lookups"] == K + K * K + K ** 3 + K ** 4


def test_tree_lookups_never_exceed_flat_on_distinct():
    rng = np.random.default_rng(4)
    for _ in range(10):
        M, K, n = int(rng.integers(1, 7)), int(rng.integers(1, 5)), int(rng.integers(1, 200))
        codes = rng.integers(0, K, size=(n, M)).astype(np.uint8)
        st = EncodingTree(codes).stats()
        distinct = len(np.unique(codes, axis=0))
        assert st["L2"] == distinct
        assert st["lookups"] <= M * distinct
        assert st["paper_bytes"] == 4 * n + 2 * (st["L1"] + st["L2"]) + st["sumP"]


# ---- float32 assignment (the reference of encoders that decide in float32) -------------------------

def test_encode_f32_agrees_with_float64_outside_rounding_ties():
    gm = GaussianMixture(24, 8, 1.1, (0.2, 1.0), (-4, 4), seed=21)
    xt, xb = gm.sample(1500, 1), gm.sample(4000, 2)
    M, K = 3, 64
    cb, _ = oracle.kmeans(xt, M, K, 5, oracle.kmeans_init_rows(1500, M, K, 4))
    a, b = oracle.encode(xb, cb), oracle.encode_f32(xb, cb)
    diff = np.argwhere(a != b)
    assert len(diff) <= 4          # float32 and float64 disagree only on near-ties
    for i, m in diff:
        sub = xb[i, m * 8:(m + 1) * 8].astype(np.float64)
        da = ((sub - cb[m, a[i, m]]) ** 2).sum()
        db = ((sub - cb[m, b[i, m]]) ** 2).sum()
        assert abs(da - db) <= 1e-6 * max(da, db)


def test_encode_f32_rounds_every_operation_and_breaks_ties_low():
    # one query at the origin, two dimensions.  Codeword 0 = (1, 2^-13): its squared distance 1 + 2^-26 rounds to 1
    # in float32; codeword 1 = (1, 0) is at exactly 1.  Float64 prefers codeword 1, float32 sees a tie -> index 0.
    cb = np.array([[[1.0, 2.0 ** -13], [1.0, 0.0], [2.0, 0.0]]], dtype=np.float32)
    x = np.zeros((1, 2), dtype=np.float32)
    assert oracle.encode(x, cb)[0, 0] == 1
    assert oracle.encode_f32(x, cb)[0, 0] == 0
    # identical codewords: the lower index wins in both
    cb2 = np.array([[[3.0, 3.0], [0.5, 0.5], [0.5, 0.5]]], dtype=np.float32)
    assert oracle.encode_f32(x, cb2)[0, 0] == 1 and oracle.encode(x, cb2)[0, 0] == 1


def test_encode_f32_equals_numpy_float32_definition():
    rng = np.random.default_rng(5)
    x = rng.normal(size=(300, 12)).astype(np.float32)
    cb = rng.normal(size=(2, 20, 6)).astype(np.float32)
    want = np.zeros((300, 2), dtype=np.uint8)
    for m in range(2):
        s = np.zeros((300, 20), dtype=np.float32)
        for j in range(6):                   # terms in index order, every operation rounded to float32
            d = (x[:, None, m * 6 + j] - cb[m][None, :, j]).astype(np.float32)
            s = (s + (d * d).astype(np.float32)).astype(np.float32)
        want[:, m] = s.argmin(axis=1)        # argmin returns the first minimum
    assert np.array_equal(oracle.encode_f32(x, cb), want)


# ---------------------------------------------------------------- scalar-product tables
def test_scalar_product_golden_worked_example():
    g = json.load(open(GOLD))
    cb = np.array(g["codebooks"], dtype=np.float32)
    q = np.array(g["query"], dtype=np.float32)
    codes = np.array(g["codes"], dtype=np.uint8)
    assert np.array_equal(oracle.lut_ip(q, cb), np.array(g["ip_lut"]))
    assert np.array_equal(oracle.adc_all_ip(q[None], cb, codes)[0], np.array(g["ip_values"]))
    ids, vals = oracle.search_ip(q[None], cb, codes, 3)
    assert ids[0].tolist() == g["ip_top3_ids"] and vals[0].tolist() == g["ip_top3"]


def test_scalar_product_tables_against_decoded_vectors_and_distance_tables():
    x, qs, cb, codes = _tiny(seed=5, n=200, d=12, M=3, K=8, q=7)
    xhat = oracle.decode(codes, cb).astype(np.float64)
    ip = oracle.adc_all_ip(qs, cb, codes)
    # the sum of table entries is the scalar product with the reconstruction (brute force, another routine)
    assert np.allclose(ip, qs.astype(np.float64) @ xhat.T, rtol=0, atol=1e-12)
    # polarisation ties the scalar-product tables to the (separately pinned) distance tables:
    #   ||q_m - c||^2 = ||q_m||^2 - 2 <q_m, c> + ||c||^2
    M, K, ds = cb.shape
    for q in qs:
        qn = (q.astype(np.float64).reshape(M, ds) ** 2).sum(1)[:, None]
        cn = (cb.astype(np.float64) ** 2).sum(2)
        assert np.allclose(oracle.lut(q, cb), qn - 2 * oracle.lut_ip(q, cb) + cn, rtol=0, atol=1e-11)
    # the search: a prefix of the order by (descending product, ascending id), with repeated encodings as exact ties
    ids = np.random.default_rng(1).permutation(1000)[:200].astype(np.int32)
    oi, ov = oracle.search_ip(qs, cb, codes, 25, ids)
    for j in range(len(qs)):
        order = np.lexsort((ids, -ip[j]))[:25]
        assert np.array_equal(oi[j], ids[order]) and np.array_equal(ov[j], ip[j][order])


def test_encode_f32_near_ties_tell_fused_from_unfused():
    """The near-tie inputs of the device encoder's test have the power they are used for: an assignment that forms
    t*t + s with a single rounding (a fused multiply-add, emulated here in float64 where the product is exact) differs
    from encode_f32 (one rounding per operation) on many of them, while on ordinary data the two agree."""
    from workload import near_tie_vectors
    rng = np.random.default_rng(8)
    M, K, ds = 4, 32, 16
    cb = rng.normal(size=(M, K, ds)).astype(np.float32) * 2
    def fused_assign(x):
        codes = np.zeros((len(x), M), dtype=np.uint8)
        for m in range(M):
            xs = x[:, m * ds:(m + 1) * ds]
            acc = np.zeros((len(x), K), dtype=np.float32)
            for j in range(ds):
                t = (xs[:, j, None] - cb[m][None, :, j]).astype(np.float32)
                acc = (t.astype(np.float64) * t.astype(np.float64) + acc.astype(np.float64)).astype(np.float32)
            codes[:, m] = np.argmin(acc, axis=1)
        return codes
    ties = near_tie_vectors(cb, 4000, seed=1)
    ref = oracle.encode_f32(ties, cb)
    differ = int((fused_assign(ties) != ref).sum())
    assert differ > 50, differ
    plain = rng.normal(size=(4000, M * ds)).astype(np.float32) * 2
    assert int((fused_assign(plain) != oracle.encode_f32(plain, cb)).sum()) <= 2


def test_leaf_term_golden_and_properties():
    """adc_all_term / search_term: the hand-worked example; a zero term changes nothing; a constant term shifts every
    distance and no rank; the sum equals the brute-force distance to the reconstruction plus the term."""
    g = json.load(open(GOLD))
    cb = np.array(g["codebooks"], dtype=np.float32)
    q = np.array([g["query"]], dtype=np.float32)
    codes = np.array(g["codes"], dtype=np.uint8)
    lt = g["leaf_term"]
    term = np.float32(lt["offset"]) + np.float32(lt["scale"]) * np.array(lt["bytes"], dtype=np.float32)
    assert term.tolist() == lt["terms"]
    assert oracle.adc_all_term(q, cb, codes, term)[0].tolist() == lt["distances"]
    ids, dist = oracle.search_term(q, cb, codes, term, 3)
    assert ids[0].tolist() == lt["top3_ids"] and dist[0].tolist() == lt["top3_dist"]
    rng = np.random.default_rng(12)
    cb2 = rng.normal(size=(3, 5, 2)).astype(np.float32)
    codes2 = rng.integers(0, 5, size=(40, 3)).astype(np.uint8)
    q2 = rng.normal(size=(4, 6)).astype(np.float32)
    t2 = rng.uniform(0, 3, size=40).astype(np.float32)
    plain = oracle.adc_all(q2, cb2, codes2)
    assert np.array_equal(oracle.adc_all_term(q2, cb2, codes2, np.zeros(40)), plain)
    brute = ((q2[:, None, :].astype(np.float64) - oracle.decode(codes2, cb2)[None].astype(np.float64)) ** 2).sum(-1)
    assert np.allclose(oracle.adc_all_term(q2, cb2, codes2, t2), brute + t2[None].astype(np.float64), rtol=1e-12)
    i0, d0 = oracle.search_term(q2, cb2, codes2, np.zeros(40), 7)
    i1, d1 = oracle.search_term(q2, cb2, codes2, np.full(40, 2.5), 7)
    assert np.array_equal(i0, i1) and np.allclose(d1, d0 + 2.5, rtol=1e-12)
    ri, rd = oracle.search(q2, cb2, codes2, 7)
    assert np.array_equal(i0, ri) and np.allclose(d0, rd, rtol=1e-12)
