"""GPU parity of the IVFADC path (coarse assignment, residual encoding, probe selection, list scan, top-k) against
oracle/ivfadc.py, element by element."""
import numpy as np
import pytest

import oracle
from oracle import ivfadc
from workload import GaussianMixture
from parity import REL_TOL, assert_topk_matches

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import paper_1509_05186_amd as etf  # noqa: E402


def say(*a):
    print(*a, flush=True)


class IvfProblem:
    """A database in (cell, residual code) form built by the oracle, and a context holding the same index."""

    def __init__(self, d, M, K, cells, N, Q, seed, comps=24, dup=1):
        gm = GaussianMixture(d, comps, 1.1, (0.2, 1.0), (-4.0, 4.0), seed=seed)
        xt = gm.sample(max(4 * cells, 4000), 1)
        self.x = gm.sample(N // dup, 2)
        if dup > 1:
            self.x = np.repeat(self.x, dup, axis=0)[np.random.default_rng(seed).permutation(N)]
        self.q = gm.sample(Q, 3)
        # coarse quantiser: rows of the training set (any set of distinct centroids serves the comparison)
        self.cent = np.ascontiguousarray(xt[np.random.default_rng(seed).permutation(len(xt))[:cells]])
        tc = ivfadc.coarse_assign(xt, self.cent)
        self.cb, _ = oracle.kmeans(ivfadc.residuals(xt, self.cent, tc), M, K, 3, oracle.kmeans_init_rows(len(xt), M, K, seed + 1))
        self.cells, self.codes = ivfadc.build(self.x, self.cent, self.cb)
        self.xhat = ivfadc.reconstruct(self.cent, self.cb, self.cells, self.codes)
        self.N, self.Q, self.k_cells = N, Q, cells

    def ctx(self, ids=None, **opts):
        c = etf.Context(device=0, stream=torch.cuda.current_stream().cuda_stream)
        for name, v in opts.items():
            c.set_option(name, v)
        c.pq_set_codebooks(self.cb)
        c.ivf_set_coarse(self.cent)
        c.ivf_build(self.cells, self.codes, ids)
        c.ivf_upload()
        return c

    def check(self, got_ids, got_dist, k, w, ids=None, what=""):
        """Every query against the oracle: the distances of all vectors of its probed cells (float64, to the
        reconstructions), the tie-aware top-k comparison on them, and the padding of short rows."""
        idv = np.arange(self.N) if ids is None else np.asarray(ids)
        pr = ivfadc.probes(self.q, self.cent, w)
        worst = 0.0
        for j in range(self.Q):
            inside = np.flatnonzero(np.isin(self.cells, pr[j]))
            diff = self.xhat[inside] - self.q[j].astype(np.float64)
            ref = np.einsum("ij,ij->i", diff, diff)
            n = min(k, len(inside))
            assert np.all(got_ids[j, n:] == -1) and np.all(np.isinf(got_dist[j, n:])), "%s q%d: padding" % (what, j)
            if n == 0:
                continue
            assert_topk_matches(got_ids[j, :n], got_dist[j, :n], ref, idv[inside], n, "%s q%d" % (what, j))
            pos = {int(v): i for i, v in enumerate(idv[inside])}
            r = ref[[pos[int(i)] for i in got_ids[j, :n]]]
            worst = max(worst, float(np.max(np.abs(got_dist[j, :n] - r) / np.maximum(r, 1e-30))))
        return worst


@pytest.fixture(scope="module")
def prob():
    # 1024 cells of about 60 vectors, 8 residual chunks of 4 dimensions; 150 queries = two tiles and a ragged one
    return IvfProblem(d=32, M=8, K=256, cells=1024, N=60000, Q=150, seed=31)


def test_ivf_assign_device_equals_oracle(prob):
    say("IVFADC: coarse assignment and residual encoding on the device")
    for opts in ({}, {"ivf_coarse_kernel": 1}, {"ivf_probe_slack": 10 ** 9}):   # matrix cores + rule; rule alone; every row redone
        c = etf.Context(device=0, stream=torch.cuda.current_stream().cuda_stream)
        for name, v in opts.items():
            c.set_option(name, v)
        c.pq_set_codebooks(prob.cb)
        c.ivf_set_coarse(prob.cent)
        cells, codes = c.ivf_assign_device(torch.from_numpy(prob.x).cuda())
        torch.cuda.synchronize()
        assert np.array_equal(cells.cpu().numpy(), prob.cells), opts
        assert np.array_equal(codes.cpu().numpy(), prob.codes), opts
    cells0, codes0 = c.ivf_assign_device(torch.empty((0, 32), dtype=torch.float32, device="cuda"))
    assert cells0.shape == (0,) and codes0.shape == (0, 8)


@pytest.mark.parametrize("w,k", [(1, 10), (8, 100), (64, 100), (1024, 50)])
def test_ivf_search_matches_oracle(prob, w, k):
    say("IVFADC search, w =", w, "k =", k)
    c = prob.ctx()
    ids, dist = c.ivf_search(torch.from_numpy(prob.q).cuda(), k, w)
    torch.cuda.synchronize()
    worst = prob.check(ids.cpu().numpy(), dist.cpu().numpy(), k, w, what="ivf w%d" % w)
    say("  worst relative error of a returned distance: %.3g; exact-kernel queries: %d" % (worst, c.last_fallback_count()))
    # the same lists as the oracle's search where no two candidates lie within the tolerance of each other
    oi, od = ivfadc.search(prob.q, prob.cent, prob.cb, prob.cells, prob.codes, k, w)
    got_i, got_d = ids.cpu().numpy(), dist.cpu().numpy()
    fin = np.isfinite(od)
    assert np.array_equal(np.isfinite(got_d), fin)
    assert np.all(np.abs(got_d[fin] - od[fin]) <= REL_TOL * od[fin] + 1e-8 * np.median(od[fin]))
    assert (got_i != oi).mean() < 0.02


def test_ivf_short_lists_are_padded(prob):
    say("IVFADC: k larger than the probed lists hold")
    c = prob.ctx()
    k, w = 200, 1
    ids, dist = c.ivf_search(torch.from_numpy(prob.q).cuda(), k, w)
    torch.cuda.synchronize()
    got_i, got_d = ids.cpu().numpy(), dist.cpu().numpy()
    assert (got_i == -1).any()              # about 60 vectors per cell: most rows are short
    prob.check(got_i, got_d, k, w, what="ivf short")
    oi, od = ivfadc.search(prob.q, prob.cent, prob.cb, prob.cells, prob.codes, k, w)
    assert np.array_equal(got_i == -1, oi == -1)


def test_ivf_exact_kernel_ids_and_small_candidate_lists(prob):
    say("IVFADC: explicit ids; every query through the exact kernel; candidate lists that overflow")
    ids_in = np.random.default_rng(5).permutation(10 * prob.N)[:prob.N].astype(np.int32)
    qd = torch.from_numpy(prob.q).cuda()
    k, w = 40, 16
    base = prob.ctx(ids=ids_in)
    want_i, want_d = base.ivf_search(qd, k, w)
    torch.cuda.synchronize()
    prob.check(want_i.cpu().numpy(), want_d.cpu().numpy(), k, w, ids=ids_in, what="ivf ids")
    assert base.last_fallback_count() == 0
    for opts in ({"force_fallback": 1}, {"cand_cap": 48}):
        c = prob.ctx(ids=ids_in, **opts)
        got_i, got_d = c.ivf_search(qd, k, w)
        torch.cuda.synchronize()
        assert c.last_fallback_count() > 0
        assert torch.equal(got_i, want_i) and torch.equal(got_d, want_d)


@pytest.mark.parametrize("w,k", [(1, 10), (64, 100), (1024, 50)])
def test_ivf_probe_selection_variants_agree(prob, w, k):
    say("IVFADC: probes from the matrix-core distances, from the rule alone, with a wide margin, with every row redone;",
        "the scan's bound from all lists, from the nearest one, with a second attempt; w =", w)
    qd = torch.from_numpy(prob.q).cuda()
    want_i, want_d = prob.ctx(ivf_coarse_kernel=1).ivf_search(qd, k, w)
    torch.cuda.synchronize()
    prob.check(want_i.cpu().numpy(), want_d.cpu().numpy(), k, w, what="ivf rule w%d" % w)
    for opts in ({}, {"ivf_probe_slack": 3000}, {"ivf_probe_slack": 10 ** 9}, {"ivf_probe_cap": 1},
                 {"ivf_bound_factor": 0}, {"ivf_bound_factor": 1}, {"ivf_bound_factor": 1, "cand_cap": 128},
                 {"ivf_coarse_tile": 0}):
        c = prob.ctx(**opts)
        got_i, got_d = c.ivf_search(qd, k, w)
        torch.cuda.synchronize()
        assert torch.equal(got_i, want_i) and torch.equal(got_d, want_d), opts


def test_ivf_probe_selection_odd_shapes():
    say("IVFADC: dimension not a multiple of 16 or 4, cells not a multiple of 32, far-off data (large norms, small distances)")
    for d, M, cells, shift in ((20, 4, 77, 0.0), (18, 6, 300, 50.0), (128, 8, 520, 0.0)):
        p = IvfProblem(d=d, M=M, K=16, cells=cells, N=5000, Q=130, seed=40 + d)
        if shift:
            p.x += np.float32(shift); p.q += np.float32(shift); p.cent += np.float32(shift)
            p.cells, p.codes = ivfadc.build(p.x, p.cent, p.cb)
            p.xhat = ivfadc.reconstruct(p.cent, p.cb, p.cells, p.codes)
        k, w = 20, 9
        qd = torch.from_numpy(p.q).cuda()
        cells, codes = p.ctx().ivf_assign_device(torch.from_numpy(p.x).cuda())
        torch.cuda.synchronize()
        assert np.array_equal(cells.cpu().numpy(), p.cells) and np.array_equal(codes.cpu().numpy(), p.codes), (d, cells)
        got_i, got_d = p.ctx().ivf_search(qd, k, w)
        want_i, want_d = p.ctx(ivf_coarse_kernel=1).ivf_search(qd, k, w)
        torch.cuda.synchronize()
        assert torch.equal(got_i, want_i) and torch.equal(got_d, want_d), (d, cells)
        if not shift:
            p.check(got_i.cpu().numpy(), got_d.cpu().numpy(), k, w, what="ivf d%d" % d)


@pytest.mark.parametrize("seed", range(10))
def test_ivf_random_shapes(seed):
    """Random shapes: the default path (matrix-core distances to the centroids, bound from the nearest lists) against the
    float32 rule for every cell with the bound from all lists, bit for bit, and against the oracle."""
    rng = np.random.default_rng(1000 + seed)
    M = int(rng.choice([2, 4, 8]))
    ds = int(rng.choice([1, 2, 4, 5, 8, 16]))
    d = M * ds
    K = int(rng.choice([4, 16, 64, 256]))
    cells = int(rng.choice([5, 33, 64, 257, 1000]))
    N = int(rng.integers(cells, 40 * cells + 200))
    Q = int(rng.choice([1, 7, 64, 129]))
    w = int(rng.integers(1, min(cells, 40) + 1))
    k = int(rng.integers(1, 120))
    say("IVFADC random shape: d", d, "M", M, "K", K, "cells", cells, "N", N, "Q", Q, "w", w, "k", k)
    p = IvfProblem(d=d, M=M, K=K, cells=cells, N=N, Q=Q, seed=500 + seed, comps=6)
    qd = torch.from_numpy(p.q).cuda()
    c = p.ctx()
    cells_d, codes_d = c.ivf_assign_device(torch.from_numpy(p.x).cuda())
    torch.cuda.synchronize()
    assert np.array_equal(cells_d.cpu().numpy(), p.cells) and np.array_equal(codes_d.cpu().numpy(), p.codes)
    got_i, got_d = c.ivf_search(qd, k, w)
    want_i, want_d = p.ctx(ivf_coarse_kernel=1, ivf_bound_factor=0).ivf_search(qd, k, w)
    torch.cuda.synchronize()
    assert torch.equal(got_i, want_i) and torch.equal(got_d, want_d)
    # against the oracle's float64 distances where the three-term form keeps its relative accuracy: with very fine
    # quantisers (many codewords for one or two dimensions) a stored vector can sit so close to a query that the
    # terms cancel, which the interface documents
    if K ** (1.0 / ds) <= 16:
        p.check(got_i.cpu().numpy(), got_d.cpu().numpy(), k, w, what="ivf random %d" % seed)


def test_ivf_heavy_duplicates_and_query_batches():
    say("IVFADC: few codewords (many equal entries, exact ties), queries in several workspace batches")
    p = IvfProblem(d=16, M=4, K=4, cells=64, N=9000, Q=200, seed=33, dup=3)
    c = p.ctx(ws_cap_bytes=1 << 20)
    st = c.ivf_stats()
    assert st["entries"] < p.N and st["max_dup"] >= 3 and st["cells"] == 64
    k, w = 25, 5
    ids, dist = c.ivf_search(torch.from_numpy(p.q).cuda(), k, w)
    torch.cuda.synchronize()
    p.check(ids.cpu().numpy(), dist.cpu().numpy(), k, w, what="ivf dups")


def test_ivf_error_paths(prob):
    c = etf.Context(device=0, stream=torch.cuda.current_stream().cuda_stream)
    c.pq_set_codebooks(prob.cb)
    qd = torch.from_numpy(prob.q).cuda()
    with pytest.raises(etf.EtfError):           # no coarse quantiser yet
        c.ivf_build(prob.cells, prob.codes)
    c.ivf_set_coarse(prob.cent)
    with pytest.raises(etf.EtfError):           # search before build
        c.ivf_search(qd, 10, 4)
    bad = prob.cells.copy()
    bad[7] = prob.k_cells
    with pytest.raises(etf.EtfError):
        c.ivf_build(bad, prob.codes)
    c.ivf_build(prob.cells, prob.codes)
    with pytest.raises(etf.EtfError):           # not uploaded
        c.ivf_search(qd, 10, 4)
    c.ivf_upload()
    for k, w in ((0, 4), (10, 0), (10, prob.k_cells + 1), (2000, 4)):
        with pytest.raises(etf.EtfError):
            c.ivf_search(qd, k, w)
