"""GPU parity: every entry point of the C ABI against the CPU oracle, element by element."""
import numpy as np
import pytest

import oracle
from workload import GaussianMixture
from parity import assert_distances_close, assert_topk_matches

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import paper_1509_05186_amd as etf  # noqa: E402

FLAT, TREE, FOREST = etf.ETF_MODE_FLAT, etf.ETF_MODE_TREE, etf.ETF_MODE_FOREST


def say(*a):
    print(*a, flush=True)


class Problem:
    def __init__(self, d, M, K, N, Q, ntrain, seed, comps=16, iters=4, dup_factor=1):
        gm = GaussianMixture(d, comps, 1.1, (0.2, 1.0), (-4.0, 4.0), seed=seed)
        xt = gm.sample(ntrain, 1)
        self.xb = gm.sample(N // dup_factor, 2)
        if dup_factor > 1:
            self.xb = np.repeat(self.xb, dup_factor, axis=0)[np.random.default_rng(seed).permutation(N)]
        self.q = gm.sample(Q, 3)
        self.cb, _ = oracle.kmeans(xt, M, K, iters, oracle.kmeans_init_rows(ntrain, M, K, seed))
        self.codes = oracle.encode(self.xb, self.cb)
        self.d, self.M, self.K, self.N, self.Q = d, M, K, N, Q
        self._all = None

    @property
    def ref_all(self):
        if self._all is None:
            self._all = oracle.adc_all(self.q, self.cb, self.codes)
        return self._all

    def ctx(self, T=1, ids=None, chunk_begin=None, **opts):
        c = etf.Context(device=0, stream=torch.cuda.current_stream().cuda_stream)
        for name, v in opts.items():
            c.set_option(name, v)
        c.pq_set_codebooks(self.cb)
        c.index_build(self.codes, ids=ids, T=T, chunk_begin=chunk_begin)
        c.index_upload()
        return c


@pytest.fixture(scope="module")
def small():
    # several tiles of queries with a ragged tail (150 = 64 + 64 + 22), K = 256, 8 chunks
    return Problem(d=32, M=8, K=256, N=20000, Q=150, ntrain=4000, seed=11)


@pytest.fixture(scope="module")
def dups():
    # few codewords => many identical encodings and exact distance ties
    return Problem(d=16, M=4, K=4, N=6000, Q=70, ntrain=500, seed=12, dup_factor=3)


def qdev(p):
    return torch.from_numpy(p.q).cuda()


# 0: matrix cores (+ exact recomputation of small entries), as workgroups of one wave (default) or of four; 1: plain sums
@pytest.mark.parametrize("lut_kernel,opts", [(0, {}), (0, {"lut_narrow_below": 1}), (1, {})])
def test_lut_build(small, lut_kernel, opts):
    say("lut_build small, kernel", lut_kernel, opts)
    c = small.ctx(lut_kernel=lut_kernel, **opts)
    lut = c.lut_build(qdev(small)).cpu().numpy()
    if opts:   # the two launch shapes of the matrix-core kernel give the same tables, bit for bit
        assert np.array_equal(lut, small.ctx(lut_kernel=lut_kernel).lut_build(qdev(small)).cpu().numpy())
    ref = np.stack([oracle.lut(q, small.cb) for q in small.q])
    assert lut.min() >= 0.0
    assert_distances_close(lut.reshape(small.Q, -1), ref.reshape(small.Q, -1), "lut kernel %d" % lut_kernel)
    say("  worst relative error of an entry: %.3g" % float((np.abs(lut - ref) / np.maximum(ref, 1e-30)).max()))


def test_lut_kernels_on_wide_subspaces():
    say("lut_build with 120-dimensional groups (odd sizes, padding), both kernels")
    p = Problem(d=7 * 17, M=7, K=50, N=500, Q=70, ntrain=600, seed=15)         # ds = 17: padded to 18 for the matrix cores
    ref = np.stack([oracle.lut(q, p.cb) for q in p.q])
    for lk in (0, 1):
        c = p.ctx(lut_kernel=lk)
        lut = c.lut_build(qdev(p)).cpu().numpy()
        assert_distances_close(lut.reshape(p.Q, -1), ref.reshape(p.Q, -1), "lut kernel %d" % lk)
        d = c.adc(qdev(p), TREE)
        torch.cuda.synchronize()
        assert_distances_close(d.cpu().numpy(), p.ref_all, "adc with lut kernel %d" % lk)


TRAVERSALS = [0, 1, 2]   # 0: distance context in registers, 1: level-synchronous kernels, 2: searches with all tables in LDS
ADC_TRAVERSALS = TRAVERSALS


@pytest.mark.parametrize("trav", ADC_TRAVERSALS)
@pytest.mark.parametrize("mode,T", [(FLAT, 1), (TREE, 1), (FOREST, 1), (FOREST, 2), (FOREST, 4), (FOREST, 8)])
def test_adc_all_pairs(small, mode, T, trav):
    if mode == FLAT and trav == 1:
        pytest.skip("flat mode has no tree traversal")
    say("adc all pairs mode", mode, "T", T, "traversal", trav)
    c = small.ctx(T=T, traversal=trav)
    dist = c.adc(qdev(small), mode)
    torch.cuda.synchronize()
    assert_distances_close(dist.cpu().numpy(), small.ref_all, "adc mode %d T %d" % (mode, T))


@pytest.mark.parametrize("trav", ADC_TRAVERSALS)
def test_tree_equals_flat_bitwise(small, trav):
    say("tree == flat bitwise, traversal", trav)
    c = small.ctx(T=1, traversal=trav)
    a = c.adc(qdev(small), FLAT)
    b = c.adc(qdev(small), TREE)
    torch.cuda.synchronize()
    assert torch.equal(a, b)       # the same float32 sum, associated the same way, shared prefixes added once


@pytest.mark.parametrize("trav", ADC_TRAVERSALS)
def test_adc_unequal_groups_and_batches(small, trav):
    say("adc unequal chunk groups, tiny workspace cap => several query batches, traversal", trav)
    c = small.ctx(T=3, chunk_begin=[0, 1, 4, 8], ws_cap_bytes=1 << 20, traversal=trav)
    dist = c.adc(qdev(small), FOREST)
    torch.cuda.synchronize()
    assert_distances_close(dist.cpu().numpy(), small.ref_all, "adc T=3")


def assert_lists_agree(a, b, what):
    """Two traversals that associate the float32 sums differently (left to right / in pairs): the distance lists
    agree to rounding, and the id lists wherever the neighbouring distances are not within rounding of each other."""
    (ai, ad), (bi, bd) = a, b
    assert np.allclose(ad, bd, rtol=2e-6, atol=0.0), what
    differ = ai != bi
    if differ.any():
        gap_next = np.abs(np.diff(ad, axis=1, append=ad[:, -1:] * 2 + 1))
        gap_prev = np.abs(np.diff(ad, axis=1, prepend=ad[:, :1] * 0 - 1))
        near_tie = np.minimum(gap_next, gap_prev) <= 4e-6 * np.abs(ad)
        last = np.zeros_like(differ)
        last[:, -1] = True                      # the k-th place can trade with the (k+1)-th, which the list does not show
        assert (near_tie | last)[differ].all(), what
        assert differ.mean() < 0.01, what


def check_search(p, c, mode, k, ids=None, what=""):
    oi, od = c.search(qdev(p), k, mode)
    torch.cuda.synchronize()
    oi, od = oi.cpu().numpy(), od.cpu().numpy()
    idv = np.arange(p.N) if ids is None else ids
    for j in range(p.Q):
        assert_topk_matches(oi[j], od[j], p.ref_all[j], idv, k, "%s q%d" % (what, j))
    return oi, od


@pytest.mark.parametrize("trav", TRAVERSALS)
@pytest.mark.parametrize("mode,T", [(FLAT, 1), (TREE, 1), (FOREST, 2), (FOREST, 4)])
@pytest.mark.parametrize("k", [1, 10, 100])
def test_search(small, mode, T, k, trav):
    if mode == FLAT and trav == 1:
        pytest.skip("flat mode has no tree traversal")
    say("search mode", mode, "T", T, "k", k, "traversal", trav)
    c = small.ctx(T=T, sample_min=2048, traversal=trav)   # small sample so that the threshold path is exercised
    check_search(small, c, mode, k, what="search m%d T%d k%d" % (mode, T, k))
    assert c.last_fallback_count() == 0


@pytest.mark.parametrize("filt", [1, 2])
@pytest.mark.parametrize("mode,T,k", [(TREE, 1, 1), (TREE, 1, 100), (FOREST, 2, 10), (FOREST, 2, 1000), (FOREST, 4, 100), (FLAT, 1, 100)])
def test_search_fixed_point_filter(small, dups, mode, T, k, filt):
    """Option lds_filter = 1 / 2: the main pass selects candidates by integer sums of scaled table entries (32-bit /
    16-bit); what is returned are float32 sums recomputed from the float32 tables, held to the same bar as every
    other search, and bit-identical to the float32 filter's results."""
    say("search with the fixed-point candidate filter", filt, "mode", mode, "T", T, "k", k)
    c = small.ctx(T=T, sample_min=2048, lds_filter=filt)
    oi, od = check_search(small, c, mode, k, what="fixed-point m%d T%d k%d" % (mode, T, k))
    assert c.last_fallback_count() == 0
    f = small.ctx(T=T, sample_min=2048, lds_filter=0)
    fi, fd = f.search(qdev(small), k, mode)
    torch.cuda.synchronize()
    assert np.array_equal(od, fd.cpu().numpy()) and np.array_equal(oi, fi.cpu().numpy())
    if k <= 100 and mode != FLAT:      # many equal encodings and exact ties
        cd = dups.ctx(T=T if T <= 2 else 2, sample_min=512, lds_filter=filt)
        check_search(dups, cd, mode if T <= 2 else FOREST, min(k, 50), what="fixed-point dups")


@pytest.mark.parametrize("context", [0, 1])
@pytest.mark.parametrize("M", [8, 16])
def test_search_sixteen_bit_filter_shapes(small, M, context):
    """The 16-bit filter kernel in both of its shapes (8 chunks: rows of 64 bytes; 16 chunks: rows of 32 bytes, two-word
    records), with and without its distance context: the bar of every other search, and the float32 filter's bits."""
    say("16-bit candidate filter, M", M, "context", context)
    p = small if M == 8 else Problem(d=32, M=16, K=256, N=20000, Q=150, ntrain=4000, seed=15)
    for T, k in ((1, 10), (M // 4, 100)):
        c = p.ctx(T=T, sample_min=2048, lds_filter=2, lds16_context=context)
        mode = TREE if T == 1 else FOREST
        c.profile_enable(True)
        oi, od = check_search(p, c, mode, k, what="16-bit filter M%d T%d ctx%d" % (M, T, context))
        assert c.last_fallback_count() == 0
        assert c.profile_read()["lds16"][1] > 0          # the kernel this test is about did run
        f = p.ctx(T=T, sample_min=2048, lds_filter=0)
        fi, fd = f.search(torch.from_numpy(p.q).cuda(), k, mode)
        torch.cuda.synchronize()
        assert np.array_equal(od, fd.cpu().numpy()) and np.array_equal(oi, fi.cpu().numpy())


@pytest.mark.parametrize("mode,T", [(FLAT, 1), (FOREST, 2)])
def test_search_large_k(small, mode, T):
    say("search with k near the maximum (largest selection buffers), mode", mode)
    c = small.ctx(T=T, sample_min=2048)
    check_search(small, c, mode, 1000, what="large k m%d" % mode)
    check_search(small, c, mode, 1024, what="max k m%d" % mode)
    assert c.last_fallback_count() == 0


def test_search_matches_oracle_lists_exactly(small):
    say("search ids identical to the oracle's (no near-ties expected at this size)")
    c = small.ctx(T=2, sample_min=2048)
    oi, od = c.search(qdev(small), 20, FOREST)
    torch.cuda.synchronize()
    ri, rd = oracle.search(small.q, small.cb, small.codes, 20)
    same = (oi.cpu().numpy() == ri).all(axis=1).mean()
    assert same > 0.9, same


@pytest.mark.parametrize("mode,T", [(FLAT, 1), (TREE, 1), (FOREST, 2)])
def test_search_exact_kernel(small, mode, T):
    say("search through the exact whole-database kernel, mode", mode)
    for trav in TRAVERSALS:      # the exact kernel associates the sums as the traversal it stands in for
        c = small.ctx(T=T, force_fallback=1, traversal=trav)
        a_i, a_d = check_search(small, c, mode, 50, what="exact m%d" % mode)
        assert c.last_fallback_count() == small.Q
        c2 = small.ctx(T=T, sample_min=2048, traversal=trav)
        b_i, b_d = c2.search(qdev(small), 50, mode)
        torch.cuda.synchronize()
        assert np.array_equal(a_i, b_i.cpu().numpy()) and np.array_equal(a_d, b_d.cpu().numpy())


@pytest.mark.parametrize("trav", TRAVERSALS)
@pytest.mark.parametrize("mode,T", [(FLAT, 1), (TREE, 1), (FOREST, 2), (FOREST, 4)])
def test_search_with_duplicates_and_custom_ids(dups, mode, T, trav):
    if mode == FLAT and trav == 1:
        pytest.skip("flat mode has no tree traversal")
    say("search on heavily duplicated encodings, custom ids, mode", mode, "traversal", trav)
    ids = (np.random.default_rng(0).permutation(dups.N) * 7 + 3).astype(np.int32)
    c = dups.ctx(T=T, ids=ids, sample_min=512, traversal=trav)
    st = c.index_stats()
    assert st["max_dup"] >= 3 and st["n_distinct"] <= 256
    for k in (1, 5, 100, 1000):
        oi, od = check_search(dups, c, mode, k, ids=ids, what="dups m%d k%d" % (mode, k))
        ri, rd = oracle.search(dups.q, dups.cb, dups.codes, k, ids)
        # both sides order exact ties by id, so the lists agree wherever float32 and float64 agree on ties
        agree = (oi == ri).all(axis=1).mean()
        assert agree > 0.8, (k, agree)


@pytest.fixture(scope="module")
def wide():
    # 16 chunks: two-word records, depth classes 16 (single tree), 8 and 4
    return Problem(d=32, M=16, K=64, N=12000, Q=70, ntrain=3000, seed=14)


@pytest.mark.parametrize("trav", TRAVERSALS)
@pytest.mark.parametrize("mode,T,cbeg", [(TREE, 1, None), (FOREST, 2, None), (FOREST, 4, None), (FOREST, 3, [0, 5, 10, 16]),
                                        (FOREST, 2, [0, 3, 16]), (FLAT, 1, None), (FOREST, 8, None), (FOREST, 16, None)])
def test_sixteen_chunks(wide, mode, T, cbeg, trav):
    if mode == FLAT and trav == 1:
        pytest.skip("flat mode has no tree traversal")
    say("M=16 mode", mode, "T", T, "chunks", cbeg, "traversal", trav)
    c = wide.ctx(T=T, chunk_begin=cbeg, sample_min=1024, traversal=trav)
    d = c.adc(qdev(wide), mode)
    torch.cuda.synchronize()
    assert_distances_close(d.cpu().numpy(), wide.ref_all, "M16 adc")
    check_search(wide, c, mode, 20, what="M16 search")


def test_search_small_database():
    say("search with N below one tile and k == N")
    p = Problem(d=8, M=2, K=8, N=40, Q=5, ntrain=100, seed=13)
    for mode, T in [(FLAT, 1), (TREE, 1), (FOREST, 2)]:
        c = p.ctx(T=T)
        check_search(p, c, mode, 40, what="tiny m%d" % mode)
        d = c.adc(qdev(p), mode)
        torch.cuda.synchronize()
        assert_distances_close(d.cpu().numpy(), p.ref_all, "tiny adc")


@pytest.mark.parametrize("M,K,N,Q", [(4, 8, 17, 3), (8, 256, 1, 1), (16, 200, 33, 70), (8, 16, 64, 64)])
def test_search_tiny_databases_through_the_lds_kernels(M, K, N, Q):
    say("tiny database through the LDS-resident kernels: M", M, "K", K, "N", N, "Q", Q)
    p = Problem(d=M * 2, M=M, K=K, N=N, Q=Q, ntrain=max(2 * K, 100), seed=31 + M, iters=2)
    for mode, T in [(FLAT, 1), (TREE, 1), (FOREST, 2), (FOREST, 4)]:
        c = p.ctx(T=T)
        for k in sorted({1, min(N, 7), N}):
            check_search(p, c, mode, k, what="tiny lds m%d T%d k%d" % (mode, T, k))
        d = c.adc(qdev(p), mode)
        torch.cuda.synchronize()
        assert_distances_close(d.cpu().numpy(), p.ref_all, "tiny lds adc")


def test_search_several_batches(small):
    say("search with a workspace cap that forces several query batches")
    c = small.ctx(T=2, sample_min=2048, ws_cap_bytes=8 << 20)
    assert c.workspace_bytes(small.Q, 10, FOREST) <= 16 << 20
    check_search(small, c, FOREST, 10, what="batched")


def test_device_error_paths(small):
    say("device entry points reject bad arguments before launching")
    lib = etf.load_library()
    c = small.ctx(T=2)
    q = qdev(small)
    ws = c.alloc_workspace(small.Q, 10, FOREST)
    oi = torch.empty((small.Q, 10), dtype=torch.int32, device="cuda")
    od = torch.empty((small.Q, 10), dtype=torch.float32, device="cuda")
    p, n = c._ws(ws)
    assert lib.etf_search(c._h, q.data_ptr(), small.Q, 10, TREE, oi.data_ptr(), od.data_ptr(), p, n) == -2
    assert lib.etf_search(c._h, q.data_ptr(), small.Q, 10, FOREST, oi.data_ptr(), od.data_ptr(), p, 1024) == -3
    assert lib.etf_search(c._h, q.data_ptr(), small.Q, 0, FOREST, oi.data_ptr(), od.data_ptr(), p, n) == -1
    assert lib.etf_search(c._h, None, small.Q, 10, FOREST, oi.data_ptr(), od.data_ptr(), p, n) == -1
    assert lib.etf_search(c._h, q.data_ptr(), small.Q, 10, FOREST, oi.data_ptr(), od.data_ptr(), p + 4, n - 4) == -1
    c2 = etf.Context(device=0)
    c2.pq_set_codebooks(small.cb)
    c2.index_build(small.codes)
    assert lib.etf_search(c2._h, q.data_ptr(), small.Q, 10, FLAT, oi.data_ptr(), od.data_ptr(), p, n) == -2  # no upload
    torch.cuda.synchronize()


@pytest.mark.parametrize("seed", [101, 102, 103, 104, 105, 106])
def test_search_random_shapes_all_traversals_agree(seed):
    """Random shapes around the limits of the LDS-resident kernel (M in {4, 8, 16}, T in {1, 2, 4}, any K): every
    traversal matches the oracle, and they agree with one another (to the bit where the sums are associated alike)."""
    rng = np.random.default_rng(seed)
    M = int(rng.choice([4, 8, 16]))
    T = int(rng.choice([t for t in (1, 2, 4) if t <= M]))
    K = int(rng.choice([2, 5, 16, 64, 200, 256]))
    ds = int(rng.choice([1, 2, 3]))
    N = int(rng.integers(300, 9000))
    Q = int(rng.integers(1, 140))
    k = int(rng.integers(1, min(N, 120)))
    dup = int(rng.choice([1, 1, 4]))
    say("random shape seed", seed, "M", M, "T", T, "K", K, "ds", ds, "N", N, "Q", Q, "k", k, "dup", dup)
    p = Problem(d=M * ds, M=M, K=K, N=N - N % dup, Q=Q, ntrain=max(4 * K, 300), seed=seed, iters=2, dup_factor=dup)
    lists = []
    for trav in TRAVERSALS:
        c = p.ctx(T=T, sample_min=256, traversal=trav)
        oi, od = check_search(p, c, FOREST, k, what="random seed %d trav %d" % (seed, trav))
        lists.append((oi, od))
    # traversals 0 and 1 add left to right: identical bits; traversal 2 adds the chunks of a group in pairs
    assert np.array_equal(lists[0][0], lists[1][0]) and np.array_equal(lists[0][1], lists[1][1])
    assert_lists_agree(lists[0], lists[2], "random seed %d: traversal 2 against 0" % seed)
    c = p.ctx(T=1, sample_min=256)
    check_search(p, c, FLAT, k, what="random seed %d flat" % seed)


def test_search_with_a_huge_group_of_repeated_vectors():
    """Two thirds of the database are copies of one vector.  The tree modes carry them as one encoding with an id
    range; the flat scan lists every copy at or below the bound, so its candidate lists must hold them all."""
    say("200000 copies of one vector among 300000")
    p = Problem(d=32, M=8, K=256, N=100000, Q=70, ntrain=4000, seed=17)
    rng = np.random.default_rng(17)
    p.codes = np.concatenate([p.codes, np.repeat(p.codes[:1], 200000, axis=0)])[rng.permutation(300000)]
    p.N = 300000
    p._all = None
    for mode, T in [(FLAT, 1), (TREE, 1), (FOREST, 2)]:
        c = p.ctx(T=T)
        assert c.index_stats()["max_dup"] >= 200000
        check_search(p, c, mode, 100, what="huge group m%d" % mode)
        assert c.last_fallback_count() == 0, mode


@pytest.mark.parametrize("mode,T", [(FLAT, 1), (FOREST, 2)])
def test_workgroup_count_does_not_change_results(small, mode, T):
    say("search and all pairs with 1, 3, 7 and the library's choice of workgroups per sub-tile, mode", mode)
    p = small
    ref = None
    for blocks in (0, 1, 3, 7):
        c = p.ctx(T=T, sample_min=2048, lds_blocks=blocks)
        oi, od = c.search(qdev(p), 50, mode)
        dist = c.adc(qdev(p), mode)
        torch.cuda.synchronize()
        got = (oi.clone(), od.clone(), dist.clone())
        if ref is None:
            ref = got
            check_search(p, c, mode, 50, what="lds_blocks")
        else:
            assert all(torch.equal(a, b) for a, b in zip(ref, got)), blocks


@pytest.mark.parametrize("trav", TRAVERSALS)
def test_forest_of_single_chunk_trees(small, trav):
    say("eight trees of one chunk each (M = 8), traversal", trav)
    c = small.ctx(T=8, sample_min=2048, traversal=trav)
    d = c.adc(qdev(small), FOREST)
    torch.cuda.synchronize()
    assert_distances_close(d.cpu().numpy(), small.ref_all, "T=8 adc")
    check_search(small, c, FOREST, 100, what="T=8 search")
    assert c.last_fallback_count() == 0
    if trav == 2:   # one- and two-chunk trees are summed like trees of four chunks: the same bits as T = 2
        c2 = small.ctx(T=2, sample_min=2048, traversal=2)
        assert torch.equal(d, c2.adc(qdev(small), FOREST))


@pytest.mark.parametrize("N", [63, 64, 65, 127, 129, 1001, 1002, 1003, 1004, 4099])
def test_all_pairs_ragged_database_sizes(N):
    """All-pairs output where the database size is, or is not, a multiple of the 4 positions a lane writes at once and of
    the 64 a wave takes per round (rows of the output 16-byte aligned or not)."""
    say("all pairs, N =", N)
    p = Problem(d=16, M=8, K=32, N=N, Q=70, ntrain=400, seed=40 + N % 7, iters=2)
    for mode, T in [(FLAT, 1), (TREE, 1), (FOREST, 2)]:
        c = p.ctx(T=T)
        d = c.adc(qdev(p), mode)
        torch.cuda.synchronize()
        assert_distances_close(d.cpu().numpy(), p.ref_all, "ragged N=%d mode %d" % (N, mode))
    # an output buffer that is not 16-byte aligned
    raw = torch.empty(p.Q * N + 1, dtype=torch.float32, device="cuda")
    out = raw[1:].view(p.Q, N)
    c.adc(qdev(p), FOREST, dist=out)
    torch.cuda.synchronize()
    assert_distances_close(out.cpu().numpy(), p.ref_all, "unaligned output")
