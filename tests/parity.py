"""Comparison helpers shared by the GPU parity tests, the smoke check and the benchmark."""
import numpy as np

REL_TOL = 1e-5          # relative tolerance on float32 distances against the float64 oracle


def dist_tol(ref):
    """|gpu - oracle| <= 1e-5 * |oracle|, with an absolute floor tied to the typical distance of the
    query for the degenerate case of an oracle distance of (almost) zero."""
    ref = np.asarray(ref, dtype=np.float64)
    floor = 1e-8 * np.median(np.abs(ref)) if ref.size else 0.0
    return REL_TOL * np.abs(ref) + floor


def assert_distances_close(gpu, ref, what=""):
    gpu = np.asarray(gpu, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert gpu.shape == ref.shape, (what, gpu.shape, ref.shape)
    err = np.abs(gpu - ref)
    tol = REL_TOL * np.abs(ref) + 1e-8 * np.median(np.abs(ref), axis=-1, keepdims=True)
    bad = err > tol
    assert not bad.any(), "%s: %d of %d distances off, worst relative error %.3g" % (
        what, int(bad.sum()), bad.size, float((err / np.maximum(np.abs(ref), 1e-300)).max()))


def assert_topk_matches(gpu_ids, gpu_dist, ref_all, ids, k, what=""):
    """Tie-aware check of one query's top-k against the oracle's distances to every vector.

    ref_all[n] is the oracle distance of input position n, ids[n] its id.  Required:
      - k distinct, valid ids, ordered ascending by (returned distance, id);
      - each returned distance agrees with the oracle distance of the returned id;
      - the returned distances agree, position by position, with the oracle's sorted top-k;
      - nothing left out is closer (beyond the tolerance) than the last one returned;
      - outside the tolerance band around the k-th distance the id lists are identical.
    """
    gpu_ids = np.asarray(gpu_ids).astype(np.int64)
    gpu_dist = np.asarray(gpu_dist, dtype=np.float64)
    ref_all = np.asarray(ref_all, dtype=np.float64)
    ids = np.asarray(ids).astype(np.int64)
    assert gpu_ids.shape == (k,) and gpu_dist.shape == (k,), what
    assert len(set(gpu_ids.tolist())) == k, what + ": duplicate ids"
    pos_of = {int(v): i for i, v in enumerate(ids)}
    assert all(int(i) in pos_of for i in gpu_ids), what + ": unknown id"
    # ordering by (distance, id)
    for a in range(k - 1):
        assert (gpu_dist[a], gpu_ids[a]) < (gpu_dist[a + 1], gpu_ids[a + 1]), what + ": order at %d" % a
    tol_all = dist_tol(ref_all)
    pos = np.array([pos_of[int(i)] for i in gpu_ids])
    assert np.all(np.abs(gpu_dist - ref_all[pos]) <= tol_all[pos]), what + ": returned distance vs oracle"
    order = np.lexsort((ids, ref_all))
    ref_top = ref_all[order[:k]]
    assert np.all(np.abs(gpu_dist - ref_top) <= dist_tol(ref_all)[order[:k]] + 1e-300), what + ": sorted distances"
    kth = ref_top[-1]
    band = REL_TOL * abs(kth) * 2 + 1e-8 * np.median(np.abs(ref_all))
    left_out = np.ones(len(ids), dtype=bool)
    left_out[pos] = False
    assert not np.any(ref_all[left_out] < kth - band), what + ": a closer vector was left out"
    # identical ids where the order is unambiguous
    sure = np.abs(ref_top - kth) > band
    for a in np.flatnonzero(sure):
        lo, hi = ref_top[a] - band, ref_top[a] + band
        clash = np.count_nonzero((ref_all >= lo) & (ref_all <= hi)) > 1
        if not clash:
            assert gpu_ids[a] == ids[order[a]], what + ": id at rank %d" % a


def assert_topk_matches_identity(gpu_ids, gpu_dist, ref_all, k, what=""):
    """The same requirements as assert_topk_matches for ids = input positions (id n is position n), written
    without per-id dictionaries or a sort of the whole array, for databases of 10^7..10^8 vectors: everything
    that can matter lies at or below the k-th oracle distance plus the tolerance band, a set found with one
    partition."""
    gpu_ids = np.asarray(gpu_ids).astype(np.int64)
    gpu_dist = np.asarray(gpu_dist, dtype=np.float64)
    ref_all = np.asarray(ref_all, dtype=np.float64)
    n = ref_all.shape[0]
    assert gpu_ids.shape == (k,) and gpu_dist.shape == (k,), what
    assert len(np.unique(gpu_ids)) == k, what + ": duplicate ids"
    assert gpu_ids.min() >= 0 and gpu_ids.max() < n, what + ": unknown id"
    for a in range(k - 1):
        assert (gpu_dist[a], gpu_ids[a]) < (gpu_dist[a + 1], gpu_ids[a + 1]), what + ": order at %d" % a
    floor = 1e-8 * float(np.median(np.abs(ref_all)))
    tol = lambda v: REL_TOL * np.abs(v) + floor
    assert np.all(np.abs(gpu_dist - ref_all[gpu_ids]) <= tol(ref_all[gpu_ids])), what + ": returned distance vs oracle"
    kth = float(np.partition(ref_all, k - 1)[k - 1])
    band = REL_TOL * abs(kth) * 2 + floor
    near = np.flatnonzero(ref_all <= kth + 2 * band)          # every position that can appear or clash
    order = near[np.lexsort((near, ref_all[near]))]
    ref_top = ref_all[order[:k]]
    assert np.all(np.abs(gpu_dist - ref_top) <= tol(ref_top) + 1e-300), what + ": sorted distances"
    closer = near[ref_all[near] < kth - band]
    assert np.all(np.isin(closer, gpu_ids)), what + ": a closer vector was left out"
    near_ref = np.sort(ref_all[near])
    for a in np.flatnonzero(np.abs(ref_top - kth) > band):
        lo, hi = ref_top[a] - band, ref_top[a] + band
        if np.searchsorted(near_ref, hi, "right") - np.searchsorted(near_ref, lo, "left") == 1:
            assert gpu_ids[a] == order[a], what + ": id at rank %d" % a


def ip_scale(lut_ip):
    """Magnitude of a query's table of scalar products: the sum over groups of the largest |entry|.  Scalar
    products cancel, so float32 results are held to 1e-5 of this scale rather than of the result itself."""
    return float(np.abs(np.asarray(lut_ip, dtype=np.float64)).max(axis=1).sum())


def assert_topk_ip_matches(gpu_ids, gpu_val, ref_all, ids, k, tol, what=""):
    """Tie-aware check of one query's k largest scalar products against the oracle's products with every vector
    (ref_all[n] for input position n, ids[n] its id), absolute tolerance tol:
      - k distinct, valid ids, ordered by (descending returned product, ascending id);
      - each returned product agrees with the oracle's for the returned id, and position by position with the
        oracle's sorted top-k;
      - nothing left out is larger (beyond the tolerance) than the last one returned;
      - where no other product lies within the tolerance band the ids are identical."""
    gpu_ids = np.asarray(gpu_ids).astype(np.int64)
    gpu_val = np.asarray(gpu_val, dtype=np.float64)
    ref_all = np.asarray(ref_all, dtype=np.float64)
    ids = np.asarray(ids).astype(np.int64)
    assert gpu_ids.shape == (k,) and gpu_val.shape == (k,), what
    assert len(set(gpu_ids.tolist())) == k, what + ": duplicate ids"
    pos_of = {int(v): i for i, v in enumerate(ids)}
    assert all(int(i) in pos_of for i in gpu_ids), what + ": unknown id"
    for a in range(k - 1):
        assert (-gpu_val[a], gpu_ids[a]) < (-gpu_val[a + 1], gpu_ids[a + 1]), what + ": order at %d" % a
    pos = np.array([pos_of[int(i)] for i in gpu_ids])
    assert np.all(np.abs(gpu_val - ref_all[pos]) <= tol), what + ": returned product vs oracle"
    order = np.lexsort((ids, -ref_all))
    ref_top = ref_all[order[:k]]
    assert np.all(np.abs(gpu_val - ref_top) <= tol), what + ": sorted products"
    kth = ref_top[-1]
    left_out = np.ones(len(ids), dtype=bool)
    left_out[pos] = False
    assert not np.any(ref_all[left_out] > kth + 2 * tol), what + ": a larger product was left out"
    for a in np.flatnonzero(np.abs(ref_top - kth) > 2 * tol):
        if np.count_nonzero(np.abs(ref_all - ref_top[a]) <= 2 * tol) == 1:
            assert gpu_ids[a] == ids[order[a]], what + ": id at rank %d" % a
