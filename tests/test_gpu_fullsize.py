"""GPU parity at the sizes of the benchmark configurations, in the launch configuration bench.py times.

The oracle cannot produce all N x Q distances of these sizes in a test, so a spread of queries (first tile,
middle tiles, the ragged last tile) is checked completely: the oracle computes their distances to every
encoding, and the tie-aware comparison of tests/parity.py is applied to the returned top-k."""
import numpy as np
import pytest

import oracle
from workload import GaussianMixture, get_config, SEED_TRAIN, SEED_DATABASE, SEED_QUERIES
from parity import assert_distances_close, assert_topk_matches, assert_topk_matches_identity

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import paper_1509_05186_amd as etf  # noqa: E402


def say(*a):
    print(*a, flush=True)


def build_inputs(cfg, N=None, Q=None):
    gm = GaussianMixture.from_config(cfg)
    N, Q = N or cfg.N, Q or cfg.Q
    host = etf.Context(device=None)
    host.pq_train(gm.sample(cfg.n_train, SEED_TRAIN), cfg.M, cfg.K, cfg.kmeans_iters, seed=SEED_TRAIN)
    codes = np.empty((N, cfg.M), dtype=np.uint8)
    done = 0
    for chunk in gm.chunks(N, SEED_DATABASE):
        codes[done:done + len(chunk)] = host.pq_encode(chunk)
        done += len(chunk)
    # these codes come from the library's host encoder: a stretch of them against the oracle's rule, so that what the
    # oracle is asked about below is what the oracle itself would have encoded
    cb = host.pq_get_codebooks()
    x0 = next(iter(gm.chunks(N, SEED_DATABASE)))[:5000]
    assert np.array_equal(oracle.encode_f32(x0, cb), codes[:len(x0)])
    return cb, codes, gm.sample(Q, SEED_QUERIES)


def make_ctx(cb, codes, T, **opts):
    c = etf.Context(device=0, stream=torch.cuda.current_stream().cuda_stream)
    for name, v in opts.items():
        c.set_option(name, v)
    c.pq_set_codebooks(cb)
    c.index_build(codes, T=T)
    c.index_upload()
    return c


def check_sampled_queries(cb, codes, queries, ids, dist, k, nsample, what):
    Q, N = queries.shape[0], codes.shape[0]
    picks = np.unique(np.concatenate([np.arange(min(4, Q)), np.linspace(0, Q - 1, nsample).astype(int), [Q - 1]]))
    for j in picks:
        ref = oracle.adc_all(queries[j:j + 1], cb, codes)[0]
        assert_topk_matches(ids[j], dist[j], ref, np.arange(N), k, "%s q%d" % (what, j))
    return len(picks)


def test_cfg2_forest_search_full_size():
    cfg = get_config("cfg2")
    say("cfg2 full size: building inputs")
    cb, codes, queries = build_inputs(cfg)
    qd = torch.from_numpy(queries).cuda()
    for trav in (0, 1, 2):
        say("cfg2 E-Forest T=2 top-100, traversal", trav)
        c = make_ctx(cb, codes, cfg.trees, traversal=trav)
        ids, dist = c.search(qd, cfg.topk, etf.ETF_MODE_FOREST)
        torch.cuda.synchronize()
        assert c.last_fallback_count() == 0
        n = check_sampled_queries(cb, codes, queries, ids.cpu().numpy(), dist.cpu().numpy(), cfg.topk, 12, "cfg2 trav%d" % trav)
        say("  checked", n, "queries against the oracle")
        if trav == 0:
            first = (ids.clone(), dist.clone())
        elif trav == 1:   # both add the chunks left to right: the same bits
            assert torch.equal(first[0], ids) and torch.equal(first[1], dist)
        else:             # the LDS-resident kernel adds the chunks of a group in pairs: equal to rounding
            assert torch.allclose(first[1], dist, rtol=2e-6, atol=0.0)
            assert (first[0] != ids).float().mean().item() < 1e-3
    say("cfg2 single E-Tree and flat, same queries")
    c = make_ctx(cb, codes, 1)
    for mode in (etf.ETF_MODE_TREE, etf.ETF_MODE_FLAT):
        ids, dist = c.search(qd, cfg.topk, mode)
        torch.cuda.synchronize()
        check_sampled_queries(cb, codes, queries, ids.cpu().numpy(), dist.cpu().numpy(), cfg.topk, 6, "cfg2 mode%d" % mode)


def test_cfg1_all_pairs_full_size():
    cfg = get_config("cfg1")
    say("cfg1 full size: all pairs, single E-Tree")
    cb, codes, queries = build_inputs(cfg)
    ref = oracle.adc_all(queries, cb, codes)
    qd = torch.from_numpy(queries).cuda()
    c = make_ctx(cb, codes, 1)
    for mode in (etf.ETF_MODE_TREE, etf.ETF_MODE_FLAT):
        d = c.adc(qd, mode)
        torch.cuda.synchronize()
        assert_distances_close(d.cpu().numpy(), ref, "cfg1 mode %d" % mode)
    c = make_ctx(cb, codes, 1, traversal=1)
    d = c.adc(qd, etf.ETF_MODE_TREE)
    torch.cuda.synchronize()
    assert_distances_close(d.cpu().numpy(), ref, "cfg1 level-synchronous")


@pytest.mark.parametrize("name,N,Q", [("cfg3", 150_000, 200), ("cfg4", 400_000, 300), ("cfg5", 600_000, 256)])
def test_other_configurations_scaled(name, N, Q):
    """Shapes of the remaining configurations (960-d vectors; 16-byte codes in 4 trees; 96-d, query batches of 256)
    at a database size the oracle can cover completely."""
    cfg = get_config(name)
    say(name, "scaled to N =", N, "Q =", Q)
    cb, codes, queries = build_inputs(cfg, N, Q)
    qd = torch.from_numpy(queries).cuda()
    ref = oracle.adc_all(queries[:40], cb, codes)
    forest = make_ctx(cb, codes, cfg.trees, sample_min=4096)
    ids, dist = forest.search(qd, cfg.topk, etf.ETF_MODE_FOREST)
    torch.cuda.synchronize()
    ids, dist = ids.cpu().numpy(), dist.cpu().numpy()
    for j in range(40):
        assert_topk_matches(ids[j], dist[j], ref[j], np.arange(N), cfg.topk, "%s forest q%d" % (name, j))
    if name == "cfg3":      # this configuration also times a single tree
        tree = make_ctx(cb, codes, 1, sample_min=4096)
        ids, dist = tree.search(qd, cfg.topk, etf.ETF_MODE_TREE)
        torch.cuda.synchronize()
        ids, dist = ids.cpu().numpy(), dist.cpu().numpy()
        for j in range(40):
            assert_topk_matches(ids[j], dist[j], ref[j], np.arange(N), cfg.topk, "cfg3 tree q%d" % j)


@pytest.mark.parametrize("name,N", [("cfg2", None), ("cfg4", 2_000_000)])
def test_device_built_index_full_size(name, N):
    """The index build on the device at the benchmark's size (cfg2) and at two million 16-byte codes in four trees
    (cfg4's shape): every array equal to the host builder's, and the same search results."""
    from test_gpu_build import assert_same_as_host_build
    cfg = get_config(name)
    say(name, "device-built index, N =", N or cfg.N)
    cb, codes, queries = build_inputs(cfg, N, 512)
    dev = etf.Context(device=0, stream=torch.cuda.current_stream().cuda_stream)
    dev.pq_set_codebooks(cb)
    img = dev.index_build_device(torch.from_numpy(codes).cuda(), T=cfg.trees)
    torch.cuda.synchronize()
    assert_same_as_host_build(dev, img, cb, codes, None, cfg.trees, None)
    host = make_ctx(cb, codes, cfg.trees)
    qd = torch.from_numpy(queries).cuda()
    a, b = dev.search(qd, cfg.topk, etf.ETF_MODE_FOREST), host.search(qd, cfg.topk, etf.ETF_MODE_FOREST)
    torch.cuda.synchronize()
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])
    assert dev.last_fallback_count() == 0
    check_sampled_queries(cb, codes, queries, a[0].cpu().numpy(), a[1].cpu().numpy(), cfg.topk, 4, name + " device-built")


def test_cfg4_forest_search_full_size():
    """cfg4 at full size (ten million 16-byte codes, four trees, ten thousand queries), in the launch configuration
    the benchmark times; the database is encoded by the device encoder (bit-identical to the oracle's float32
    assignment, see test_gpu_encode), sampled queries are checked completely against the oracle."""
    cfg = get_config("cfg4")
    gm = GaussianMixture.from_config(cfg)
    host = etf.Context(device=None)
    host.pq_train(gm.sample(cfg.n_train, SEED_TRAIN), cfg.M, cfg.K, cfg.kmeans_iters, seed=SEED_TRAIN)
    cb = host.pq_get_codebooks()
    c = etf.Context(device=0, stream=torch.cuda.current_stream().cuda_stream)
    c.pq_set_codebooks(cb)
    codes = np.empty((cfg.N, cfg.M), dtype=np.uint8)
    done = 0
    for chunk in gm.chunks(cfg.N, SEED_DATABASE):
        codes[done:done + len(chunk)] = c.pq_encode_device(torch.from_numpy(chunk).cuda()).cpu().numpy()
        done += len(chunk)
        if (done >> 17) % 16 == 0:
            say("  cfg4: generated + encoded", done, "of", cfg.N)
    queries = gm.sample(cfg.Q, SEED_QUERIES)
    qd = torch.from_numpy(queries).cuda()
    say("cfg4 full size: device build, search")
    c.index_build_device(torch.from_numpy(codes).cuda(), T=cfg.trees)
    ids, dist = c.search(qd, cfg.topk, etf.ETF_MODE_FOREST)
    torch.cuda.synchronize()
    assert c.last_fallback_count() == 0
    n = check_sampled_queries(cb, codes, queries, ids.cpu().numpy(), dist.cpu().numpy(), cfg.topk, 6, "cfg4")
    say("  checked", n, "queries against the oracle")
    say("cfg4 full size: host build, same lists")
    h = make_ctx(cb, codes, cfg.trees)
    hi, hd = h.search(qd, cfg.topk, etf.ETF_MODE_FOREST)
    torch.cuda.synchronize()
    assert torch.equal(ids, hi) and torch.equal(dist, hd)


def device_encoded_database(cfg, workers=12):
    """Codebooks trained by the library, the database encoded chunk by chunk by the device encoder (the way
    bench.py prepares every configuration): (codebooks, codes [N][M] on the host, queries)."""
    gm = GaussianMixture.from_config(cfg)
    host = etf.Context(device=None)
    host.pq_train(gm.sample(cfg.n_train, SEED_TRAIN), cfg.M, cfg.K, cfg.kmeans_iters, seed=SEED_TRAIN)
    cb = host.pq_get_codebooks()
    enc = etf.Context(device=0, stream=torch.cuda.current_stream().cuda_stream)
    enc.pq_set_codebooks(cb)
    codes = np.empty((cfg.N, cfg.M), dtype=np.uint8)
    done, step = 0, max(1, (cfg.N >> 17) // 8)
    for i, chunk in enumerate(gm.chunks_threaded(cfg.N, SEED_DATABASE, workers)):
        codes[done:done + len(chunk)] = enc.pq_encode_device(torch.from_numpy(chunk).cuda()).cpu().numpy()
        done += len(chunk)
        if i % step == 0:
            say("  %s: generated + encoded %d of %d" % (cfg.name, done, cfg.N))
    return cb, codes, gm.sample(cfg.Q, SEED_QUERIES)


def check_spread_queries(cb, codes, queries, ids, dist, k, picks, what):
    """Complete check of a few queries: the oracle's distances to every encoding, one query at a time."""
    for j in picks:
        ref = oracle.adc_all(queries[j:j + 1], cb, codes)[0]
        assert_topk_matches_identity(ids[j], dist[j], ref, k, "%s q%d" % (what, j))
        say("  %s: query %d matches the oracle" % (what, j))


def test_cfg3_tree_and_forest_full_size():
    """cfg3 at full size (d = 960, one million vectors, one thousand queries): the single E-Tree and the E-Forest of
    two trees, both of which this configuration times."""
    cfg = get_config("cfg3")
    say("cfg3 full size: inputs")
    cb, codes, queries = device_encoded_database(cfg)
    # the device encoder's decisions at 120 dimensions per group, on a spread of the database
    gm = GaussianMixture.from_config(cfg)
    first = next(gm.chunks(cfg.N, SEED_DATABASE))
    assert np.array_equal(codes[:4096], oracle.encode_f32(first[:4096], cb))
    qd = torch.from_numpy(queries).cuda()
    picks = [0, 63, 64, 500, 959, 960, cfg.Q - 1]          # first tile, a tile boundary, the ragged last tile
    for T, mode, what in ((1, etf.ETF_MODE_TREE, "cfg3 E-Tree"), (cfg.trees, etf.ETF_MODE_FOREST, "cfg3 E-Forest")):
        say(what)
        c = make_ctx(cb, codes, T)
        ids, dist = c.search(qd, cfg.topk, mode)
        torch.cuda.synchronize()
        assert c.last_fallback_count() == 0
        check_spread_queries(cb, codes, queries, ids.cpu().numpy(), dist.cpu().numpy(), cfg.topk, picks, what)


def test_cfg5_forest_search_full_size():
    """cfg5 at full size: 10^8 vectors of 96 dimensions (800 MB of codes; 16.8 million distinct encodings, one of
    them with more than a million copies), E-Forest of two trees, the thousand queries sent in calls of 256 as the
    workload defines and bench.py times; index built on the device from the device encoder's codes."""
    cfg = get_config("cfg5")
    say("cfg5 full size: inputs")
    cb, codes, queries = device_encoded_database(cfg)
    c = etf.Context(device=0, stream=torch.cuda.current_stream().cuda_stream)
    c.pq_set_codebooks(cb)
    say("cfg5: index build on the device")
    c.index_build_device(torch.from_numpy(codes).cuda(), T=cfg.trees)
    st = c.index_stats()
    say("  distinct encodings %d, largest group of equal encodings %d" % (st["n_distinct"], st["max_dup"]))
    qd = torch.from_numpy(queries).cuda()
    ids = torch.empty((cfg.Q, cfg.topk), dtype=torch.int32, device="cuda")
    dist = torch.empty((cfg.Q, cfg.topk), dtype=torch.float32, device="cuda")
    ws = c.alloc_workspace(cfg.query_batch, cfg.topk, etf.ETF_MODE_FOREST)
    fallbacks = 0
    for a in range(0, cfg.Q, cfg.query_batch):
        b = min(cfg.Q, a + cfg.query_batch)
        c.search(qd[a:b], cfg.topk, etf.ETF_MODE_FOREST, ids[a:b], dist[a:b], ws)
        fallbacks += c.last_fallback_count()
    torch.cuda.synchronize()
    assert fallbacks == 0
    picks = [0, 255, 256, 640, cfg.Q - 1]                   # both sides of a call boundary, the ragged last call
    check_spread_queries(cb, codes, queries, ids.cpu().numpy(), dist.cpu().numpy(), cfg.topk, picks, "cfg5")


def test_ivfadc_full_size():
    """IVFADC in the configuration the paper's application experiment quotes (8192 cells, w = 64, residual PQ M = 8,
    K = 256) on cfg2's vectors and all of its queries, as bench.py times it.  The database side (cells, residual codes)
    comes from the device assignment; a stretch of it is held against the oracle's assignment first, then a spread of
    queries against the oracle's distances to the reconstructions inside the oracle's probed lists."""
    from oracle import ivfadc
    cfg = get_config("cfg2")
    cells_n, w, k = 8192, 64, 100
    say("IVFADC at full size:", cfg.N, "vectors,", cells_n, "cells, w", w)
    gm = GaussianMixture.from_config(cfg)
    stream = torch.cuda.current_stream().cuda_stream
    cent = gm.sample(cells_n, 77)
    xt = gm.sample(cfg.n_train, SEED_TRAIN)
    nt = 1200                                                                    # residual codebooks from the oracle's side
    tc = ivfadc.coarse_assign(xt[:nt], cent)                                     # (its float32 rule takes 9 ms per vector here)
    cb, _ = oracle.kmeans(xt[:nt] - cent[tc], cfg.M, cfg.K, 4, oracle.kmeans_init_rows(nt, cfg.M, cfg.K, 5))
    c = etf.Context(device=0, stream=stream)
    c.pq_set_codebooks(cb)
    c.ivf_set_coarse(cent)
    cells = np.empty(cfg.N, dtype=np.int32)
    codes = np.empty((cfg.N, cfg.M), dtype=np.uint8)
    done = 0
    first = None
    for chunk in gm.chunks(cfg.N, SEED_DATABASE):
        first = chunk[:500] if first is None else first
        ce, co = c.ivf_assign_device(torch.from_numpy(chunk).cuda())
        cells[done:done + len(chunk)] = ce.cpu().numpy()
        codes[done:done + len(chunk)] = co.cpu().numpy()
        done += len(chunk)
    say("  assigned and encoded; checking a stretch against the oracle")
    oc, oe = ivfadc.build(first, cent, cb)
    assert np.array_equal(oc, cells[:len(first)]) and np.array_equal(oe, codes[:len(first)])
    c.ivf_build(cells, codes)
    c.ivf_upload()
    queries = gm.sample(cfg.Q, SEED_QUERIES)
    ids, dist = c.ivf_search(torch.from_numpy(queries).cuda(), k, w)
    torch.cuda.synchronize()
    fallbacks = c.last_fallback_count()
    ids, dist = ids.cpu().numpy(), dist.cpu().numpy()
    xhat = ivfadc.reconstruct(cent, cb, cells, codes)
    picks = [0, 1, 63, 64, 2500, 5000, 7777, cfg.Q - 1]
    pr = ivfadc.probes(queries[picks], cent, w)
    for jj, j in enumerate(picks):
        inside = np.flatnonzero(np.isin(cells, pr[jj]))
        diff = xhat[inside] - queries[j].astype(np.float64)
        ref = np.einsum("ij,ij->i", diff, diff)
        assert len(inside) >= k
        assert_topk_matches(ids[j], dist[j], ref, inside, k, "ivf full size q%d" % j)
    say("  %d queries checked; queries answered by the exact kernel: %d" % (len(picks), fallbacks))
    assert fallbacks == 0
