"""Index build on the device: the arrays against their definition (sorted distinct encodings, id ranges) and, level
arrays included, against the host builder's image (itself checked against the oracle's pointer trie), and searches /
all-pairs distances on a device-built index against the oracle and against the host-built index."""
import numpy as np
import pytest

import oracle
from parity import assert_distances_close, assert_topk_matches
from test_gpu_parity import Problem, qdev, say, FLAT, TREE, FOREST

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import paper_1509_05186_amd as etf  # noqa: E402


def dev_ctx(cb, codes, ids=None, T=1, chunk_begin=None, order=None, **opts):
    c = etf.Context(device=0, stream=torch.cuda.current_stream().cuda_stream)
    for name, v in opts.items():
        c.set_option(name, v)
    c.pq_set_codebooks(cb)
    c.index_set_chunk_order(order)
    img = c.index_build_device(torch.from_numpy(codes).cuda(), None if ids is None else torch.from_numpy(ids).cuda(),
                               T=T, chunk_begin=chunk_begin)
    torch.cuda.synchronize()
    return c, img


def arr(img, lay_off, count, dtype):
    base = (-img.data_ptr()) % 256
    nbytes = count * np.dtype(dtype).itemsize
    return img[base + lay_off: base + lay_off + nbytes].cpu().numpy().view(dtype)


def check_image(c, img, codes, ids):
    N, M = codes.shape
    st, lay = c.index_stats(), c.index_layout()
    Nd = st["n_distinct"]
    want_ecodes, inverse, counts = np.unique(codes, axis=0, return_inverse=True, return_counts=True)   # lexicographic
    assert Nd == len(want_ecodes) and st["N"] == N and st["max_dup"] == counts.max()
    idv = np.arange(N, dtype=np.int32) if ids is None else ids
    assert np.array_equal(arr(img, lay.codes, N * M, np.uint8).reshape(N, M), codes)
    assert np.array_equal(arr(img, lay.ids_in, N, np.int32), idv)
    assert np.array_equal(arr(img, lay.ecodes, Nd * M, np.uint8).reshape(Nd, M), want_ecodes)
    assert np.array_equal(arr(img, lay.enc_of_pos, N, np.uint32), inverse.reshape(-1).astype(np.uint32))
    assert np.array_equal(arr(img, lay.ebegin, Nd + 1, np.uint32), np.concatenate([[0], np.cumsum(counts)]).astype(np.uint32))
    order = np.lexsort((idv, inverse.reshape(-1)))                      # by encoding, then ascending id
    assert np.array_equal(arr(img, lay.ids_sorted, N, np.int32), idv[order])
    # the samples: distinct rows, stored once more as encodings in sample order
    se = arr(img, lay.sample_enc, lay.n_sample_enc, np.uint32)
    sp = arr(img, lay.sample_pos, lay.n_sample_pos, np.uint32)
    assert len(np.unique(se)) == len(se) and se.max() < Nd and len(np.unique(sp)) == len(sp) and sp.max() < N
    assert np.array_equal(arr(img, lay.sample_enc_codes, len(se) * M, np.uint8).reshape(-1, M), want_ecodes[se])
    assert np.array_equal(arr(img, lay.sample_pos_codes, len(sp) * M, np.uint8).reshape(-1, M), codes[sp])
    return st, lay, se, sp


def image_arrays(lay, st, M):
    """(name, offset, bytes) of every array of an index image except the threshold samples."""
    N, Nd, T = st["N"], st["n_distinct"], st["T"]
    out = [("codes", lay.codes, N * M), ("ids_in", lay.ids_in, 4 * N), ("ids_sorted", lay.ids_sorted, 4 * N),
           ("ebegin", lay.ebegin, 4 * (Nd + 1)), ("enc_of_pos", lay.enc_of_pos, 4 * N), ("ecodes", lay.ecodes, Nd * M),
           ("rec0", lay.rec0, Nd * lay.rec0_stride)]
    for t, tr in enumerate(st["trees"]):
        U = sum(tr["nL"])
        if T > 1:
            out.append(("leaf_of%d" % t, lay.leaf_of[t], 4 * Nd))
        out.append(("rec%d" % t, lay.trec[t], U * lay.trec_stride[t]))
        for l in range(tr["D"]):
            nI, nL = tr["nI"][l], tr["nL"][l]
            out += [("icode%d.%d" % (t, l), lay.icode[t][l], nI), ("iparent%d.%d" % (t, l), lay.iparent[t][l], 4 * nI),
                    ("lcodes%d.%d" % (t, l), lay.lcodes[t][l], nL * lay.lstride[t][l]),
                    ("lparent%d.%d" % (t, l), lay.lparent[t][l], 4 * nL), ("lrow%d.%d" % (t, l), lay.lrow[t][l], 4 * nL)]
    return out


def assert_same_as_host_build(c, img, cb, codes, ids, T, chunk_begin, order=None, **opts):
    """Every array of the device-built image equals the host builder's."""
    h = etf.Context(device=None)
    for name, v in opts.items():
        h.set_option(name, v)
    h.pq_set_codebooks(cb)
    h.index_set_chunk_order(order)
    h.index_build(codes, ids=ids, T=T, chunk_begin=chunk_begin)
    hs, hl, hbuf = h.index_stats(), h.index_layout(), h.index_export()
    ds, dl = c.index_stats(), c.index_layout()
    # (the host's samples are draws with repeats removed, the device's one row per stratum: their sizes differ, and
    # with them the offsets of the arrays behind them and the total)
    assert {k: v for k, v in ds.items() if k != "device_bytes"} == {k: v for k, v in hs.items() if k != "device_bytes"}
    dbuf = arr(img, 0, c.index_device_bytes(), np.uint8)
    ha, da = image_arrays(hl, hs, codes.shape[1]), image_arrays(dl, ds, codes.shape[1])
    assert [(n, b) for n, o, b in ha] == [(n, b) for n, o, b in da]
    ends = sorted(o + b for n, o, b in da)
    assert all(o >= 0 and o % 256 == 0 for n, o, b in da) and ends[-1] <= c.index_device_bytes()
    for (name, hoff, nbytes), (_, doff, _) in zip(ha, da):
        assert np.array_equal(dbuf[doff:doff + nbytes], hbuf[hoff:hoff + nbytes]), name


@pytest.mark.parametrize("N,M,K,with_ids,T,cbeg,seed", [
    (20000, 8, 256, False, 1, None, 1),          # the benchmark's code width, a single tree
    (20000, 8, 256, False, 2, None, 11),         # ... the benchmark's forest
    (5000, 8, 4, True, 4, None, 2),              # few codewords: many repeated encodings, explicit ids decide their order
    (3000, 16, 256, False, 4, None, 3),          # sixteen chunks: two sort passes
    (3000, 16, 2, True, 1, None, 4),             # ... with repeats and explicit ids: three; one tree sixteen levels deep
    (3000, 16, 3, False, 2, [0, 1, 16], 8),      # a tree of fifteen chunks: its own order takes two passes as well
    (4097, 4, 7, True, 2, None, 5),              # four chunks, K not a power of two
    (6000, 8, 5, False, 3, [0, 3, 5, 8], 9),     # unequal trees
    (1, 8, 256, False, 2, None, 6),              # a single vector
    (700, 3, 5, True, 1, None, 7),               # an odd number of chunks
    (500, 2, 9, False, 2, None, 10),             # trees of a single chunk: leaves only
])
def test_device_built_arrays(N, M, K, with_ids, T, cbeg, seed):
    say("device build arrays N", N, "M", M, "K", K, "ids", with_ids, "T", T, cbeg)
    rng = np.random.default_rng(seed)
    codes = rng.integers(0, K, size=(N, M)).astype(np.uint8)
    if K > 16:
        codes[:, : M // 2] //= 64                                          # shared prefixes and some repeats
        codes[rng.integers(0, N, N // 10)] = codes[rng.integers(0, N, N // 10)]
    ids = rng.permutation(10 * N + 5)[:N].astype(np.int32) if with_ids else None
    cb = np.zeros((M, K, 1), dtype=np.float32)
    c, img = dev_ctx(cb, codes, ids, T=T, chunk_begin=cbeg, sample_min=256)
    check_image(c, img, codes, ids)
    assert_same_as_host_build(c, img, cb, codes, ids, T, cbeg, sample_min=256)


def test_device_build_sample_sizes_and_spread():
    say("device build: sample sizes and spread on 300000 vectors")
    rng = np.random.default_rng(4)
    N, M, K = 300000, 8, 16
    codes = rng.integers(0, K, size=(N, M)).astype(np.uint8)
    codes[:, :3] //= 4
    c, img = dev_ctx(np.zeros((M, K, 1), dtype=np.float32), codes, None, T=2, sample_min=1000)
    st, lay, se, sp = check_image(c, img, codes, None)
    Nd = st["n_distinct"]
    draws = int(120 * np.sqrt(Nd))                                # the default sample_scale
    assert 0.97 * draws <= len(se) <= draws and len(sp) == int(120 * np.sqrt(N))   # repeated draws of an encoding are dropped
    # positions: one draw from each of len(sp) equal strata, in scattered order
    srt, s = np.sort(sp.astype(np.int64)), np.arange(len(sp), dtype=np.int64)
    assert np.all(srt >= s * N // len(sp)) and np.all(srt < (s + 1) * N // len(sp))
    assert np.abs(np.diff(sp.astype(np.int64))).min() > N // (4 * len(sp))
    # encodings: drawn through the vectors, so in proportion to their multiplicity: the mean multiplicity over the
    # sample is the size-biased mean sum(m^2) / N, not the plain mean N / Nd (a few hundred pairs of equal vectors here)
    enc_of_pos = arr(img, lay.enc_of_pos, N, np.uint32)
    mult = np.bincount(enc_of_pos, minlength=Nd).astype(np.float64)
    biased, plain, got = (mult ** 2).sum() / N, mult.mean(), mult[se].mean()
    assert biased - plain > 1e-3 and abs(got - biased) < abs(got - plain), (biased, plain, got)


@pytest.fixture(scope="module")
def small():
    return Problem(d=32, M=8, K=256, N=20000, Q=150, ntrain=4000, seed=11)


@pytest.mark.parametrize("trav", [0, 1, 2])
@pytest.mark.parametrize("mode,T", [(FLAT, 1), (TREE, 1), (FOREST, 2), (FOREST, 4)])
def test_search_on_device_built_index(small, mode, T, trav):
    if mode == FLAT and trav == 1:
        pytest.skip("flat mode has no tree traversal")
    say("search on a device-built index, mode", mode, "T", T, "traversal", trav)
    p = small
    c, img = dev_ctx(p.cb, p.codes, None, T=T, sample_min=2048, traversal=trav)
    h = p.ctx(T=T, sample_min=2048, traversal=trav)
    for k in (1, 100):
        oi, od = c.search(qdev(p), k, mode)
        hi, hd = h.search(qdev(p), k, mode)
        torch.cuda.synchronize()
        oi, od = oi.cpu().numpy(), od.cpu().numpy()
        for j in range(p.Q):
            assert_topk_matches(oi[j], od[j], p.ref_all[j], np.arange(p.N), k, "device-built m%d T%d q%d" % (mode, T, j))
        # same kernels, same arithmetic, another sample: identical lists
        assert np.array_equal(od, hd.cpu().numpy()) and np.array_equal(oi, hi.cpu().numpy())
        assert c.last_fallback_count() == 0
    dist = c.adc(qdev(p), mode)
    torch.cuda.synchronize()
    assert_distances_close(dist.cpu().numpy(), p.ref_all, "all pairs on a device-built index")
    assert torch.equal(dist, h.adc(qdev(p), mode))


def test_search_device_built_duplicates_ids_sixteen_chunks():
    say("device-built index: repeated encodings with explicit ids (M = 4), and M = 16")
    p = Problem(d=16, M=4, K=4, N=6000, Q=70, ntrain=500, seed=12, dup_factor=3)
    ids = np.random.default_rng(5).permutation(3 * p.N)[: p.N].astype(np.int32)
    for mode, T in [(FLAT, 1), (TREE, 1), (FOREST, 2)]:
        c, _ = dev_ctx(p.cb, p.codes, ids, T=T)
        oi, od = c.search(qdev(p), 50, mode)
        torch.cuda.synchronize()
        for j in range(p.Q):
            assert_topk_matches(oi[j].cpu().numpy(), od[j].cpu().numpy(), p.ref_all[j], ids, 50, "dups m%d q%d" % (mode, j))
    w = Problem(d=64, M=16, K=256, N=12000, Q=70, ntrain=3000, seed=13)
    c, _ = dev_ctx(w.cb, w.codes, None, T=4, sample_min=1024)
    oi, od = c.search(qdev(w), 20, FOREST)
    torch.cuda.synchronize()
    for j in range(w.Q):
        assert_topk_matches(oi[j].cpu().numpy(), od[j].cpu().numpy(), w.ref_all[j], np.arange(w.N), 20, "M16 q%d" % j)


def test_encode_then_build_then_search_all_on_the_device(small):
    say("vectors -> device encoder -> device build -> search, nothing through the host")
    p = small
    c = etf.Context(device=0, stream=torch.cuda.current_stream().cuda_stream)
    c.pq_set_codebooks(p.cb)
    codes = c.pq_encode_device(torch.from_numpy(p.xb).cuda())
    c.index_build_device(codes, T=2)
    oi, od = c.search(qdev(p), 10, FOREST)
    torch.cuda.synchronize()
    ref = oracle.adc_all(p.q, p.cb, codes.cpu().numpy())      # the float32 encoder may differ from the float64 one on near-ties
    for j in range(p.Q):
        assert_topk_matches(oi[j].cpu().numpy(), od[j].cpu().numpy(), ref[j], np.arange(p.N), 10, "all-device q%d" % j)


def test_device_build_error_paths(small):
    say("device build: error paths")
    p = small
    c = etf.Context(device=0, stream=torch.cuda.current_stream().cuda_stream)
    with pytest.raises(etf.EtfError):
        c.index_build_device_bytes(10)                                            # no codebooks
    c.pq_set_codebooks(p.cb)
    codes = torch.from_numpy(p.codes).cuda()
    nimg, nws = c.index_build_device_bytes(p.N)
    with pytest.raises(etf.EtfError):
        c.index_build_device(codes, T=3)                                          # 3 does not divide 8
    with pytest.raises(etf.EtfError):
        c.index_build_device_bytes(p.N, 3)
    with pytest.raises(etf.EtfError):
        c.index_build_device(codes, image=torch.empty(nimg // 16, dtype=torch.uint8, device="cuda"))   # fails at the first arrays
    with pytest.raises(etf.EtfError):
        c.index_build_device(codes, ws=torch.empty(nws // 2, dtype=torch.uint8, device="cuda"))
    with pytest.raises(etf.EtfError):
        c.index_build_device(codes, ids=torch.full((p.N,), -1, dtype=torch.int32, device="cuda"))
    with pytest.raises(etf.EtfError):
        c.search(qdev(p), 5, TREE)                                                # every failed build left no index
    # code bytes beyond K
    c2 = etf.Context(device=0, stream=torch.cuda.current_stream().cuda_stream)
    c2.pq_set_codebooks(np.zeros((8, 5, 1), dtype=np.float32))
    with pytest.raises(etf.EtfError):
        c2.index_build_device(torch.full((100, 8), 5, dtype=torch.uint8, device="cuda"))
    # the image the build needs is known afterwards: a buffer of exactly that size serves, one byte less fails late
    c.index_build_device(codes, T=2)
    need = c.index_device_bytes()
    assert need <= c.index_build_device_bytes(p.N, 2)[0]
    exact = torch.empty(need + 256, dtype=torch.uint8, device="cuda")
    off = (-exact.data_ptr()) % 256
    c.index_build_device(codes, T=2, image=exact[off:off + need])
    c.search(qdev(p), 5, FOREST)
    with pytest.raises(etf.EtfError):
        c.index_build_device(codes, T=2, image=exact[off:off + need - 256])
    # a device-built index has no host copy
    c.index_build_device(codes, T=2)
    with pytest.raises(etf.EtfError):
        c.index_export()
    with pytest.raises(etf.EtfError):
        c.index_upload()
