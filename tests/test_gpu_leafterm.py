"""GPU parity of the leaf payload (one additive term per vector, stored on the leaf): every distance the library
reports is the table sum plus the vector's term, in all modes and traversals, against oracle.adc_all_term."""
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


class TermProblem:
    def __init__(self, d, M, K, N, Q, seed, dup=1, levels=0):
        gm = GaussianMixture(d, 16, 1.1, (0.2, 1.0), (-4.0, 4.0), seed=seed)
        xt = gm.sample(4000, 1)
        xb = gm.sample(N // dup, 2)
        if dup > 1:
            xb = np.repeat(xb, dup, axis=0)[np.random.default_rng(seed).permutation(N)]
        self.q = gm.sample(Q, 3)
        self.cb, _ = oracle.kmeans(xt, M, K, 3, oracle.kmeans_init_rows(4000, M, K, seed))
        self.codes = oracle.encode(xb, self.cb)
        plain = oracle.adc_all(self.q[:8], self.cb, self.codes)
        rng = np.random.default_rng(seed + 1)
        scale = float(np.median(plain)) * 0.5          # large enough to reorder the neighbours
        if levels:                                      # few distinct values: equal and unequal terms on equal encodings
            self.term = (rng.integers(0, levels, size=N) * (scale / levels)).astype(np.float32)
        else:
            self.term = rng.uniform(0, scale, size=N).astype(np.float32)
        self.ref = oracle.adc_all_term(self.q, self.cb, self.codes, self.term)
        self.N, self.Q = N, Q

    def ctx(self, T=1, ids=None, term=True, **opts):
        c = etf.Context(device=0, stream=torch.cuda.current_stream().cuda_stream)
        for name, v in opts.items():
            c.set_option(name, v)
        c.pq_set_codebooks(self.cb)
        if term:
            c.index_set_leaf_term(self.term)
        c.index_build(self.codes, ids=ids, T=T)
        c.index_upload()
        return c


@pytest.fixture(scope="module")
def prob():
    return TermProblem(d=32, M=8, K=256, N=20000, Q=150, seed=41)


@pytest.fixture(scope="module")
def dups():
    return TermProblem(d=16, M=4, K=4, N=6000, Q=70, seed=42, dup=3, levels=3)


def qdev(p):
    return torch.from_numpy(p.q).cuda()


@pytest.mark.parametrize("trav", [0, 1, 2])
@pytest.mark.parametrize("mode,T", [(FLAT, 1), (TREE, 1), (FOREST, 2), (FOREST, 4)])
def test_adc_with_leaf_term(prob, mode, T, trav):
    if mode == FLAT and trav == 1:
        pytest.skip("flat mode has no tree traversal")
    say("all-pairs distances with a leaf term, mode", mode, "T", T, "traversal", trav)
    c = prob.ctx(T=T, traversal=trav)
    d = c.adc(qdev(prob), mode)
    torch.cuda.synchronize()
    assert_distances_close(d.cpu().numpy(), prob.ref, "adc term m%d T%d t%d" % (mode, T, trav))


@pytest.mark.parametrize("trav", [0, 1, 2])
@pytest.mark.parametrize("mode,T,k", [(FLAT, 1, 10), (TREE, 1, 100), (FOREST, 2, 10), (FOREST, 2, 100), (FOREST, 4, 30)])
def test_search_with_leaf_term(prob, dups, mode, T, k, trav):
    if mode == FLAT and trav == 1:
        pytest.skip("flat mode has no tree traversal")
    say("search with a leaf term, mode", mode, "T", T, "k", k, "traversal", trav)
    for p, kk, smin in ((prob, k, 2048), (dups, min(k, 40), 512)):
        TT = T if p is prob or T <= 2 else 2
        c = p.ctx(T=TT, traversal=trav, sample_min=smin)
        ids, dist = c.search(qdev(p), kk, mode)
        torch.cuda.synchronize()
        ids, dist = ids.cpu().numpy(), dist.cpu().numpy()
        for j in range(p.Q):
            assert_topk_matches(ids[j], dist[j], p.ref[j], np.arange(p.N), kk, "search term m%d T%d t%d q%d" % (mode, TT, trav, j))


def test_leaf_term_exact_kernel_ids_bytes_and_fixed_point_option(prob):
    say("leaf term: exact kernel, explicit ids, the one-byte form, option lds_filter")
    ids_in = np.random.default_rng(6).permutation(10 * prob.N)[:prob.N].astype(np.int32)
    qd = qdev(prob)
    k = 50
    base = prob.ctx(T=2, ids=ids_in, sample_min=2048)
    bi, bd = base.search(qd, k, FOREST)
    torch.cuda.synchronize()
    bi_h, bd_h = bi.cpu().numpy(), bd.cpu().numpy()
    for j in range(prob.Q):
        assert_topk_matches(bi_h[j], bd_h[j], prob.ref[j], ids_in, k, "term ids q%d" % j)
    for opts in ({"force_fallback": 1}, {"lds_filter": 1}):
        c = prob.ctx(T=2, ids=ids_in, sample_min=2048, **opts)
        gi, gd = c.search(qd, k, FOREST)
        torch.cuda.synchronize()
        assert torch.equal(gi, bi) and torch.equal(gd, bd)
    # one byte per vector: term = offset + scale * byte
    b = np.random.default_rng(7).integers(0, 256, size=prob.N).astype(np.uint8)
    scale, offset = np.float32(0.03125), np.float32(0.5)
    c = etf.Context(device=0, stream=torch.cuda.current_stream().cuda_stream)
    c.pq_set_codebooks(prob.cb)
    c.index_set_leaf_bytes(b, float(scale), float(offset))
    c.index_build(prob.codes, T=2)
    c.index_upload()
    ref = oracle.adc_all_term(prob.q, prob.cb, prob.codes, offset + scale * b.astype(np.float32))
    d = c.adc(qd, FOREST)
    gi, gd = c.search(qd, k, FOREST)
    torch.cuda.synchronize()
    assert_distances_close(d.cpu().numpy(), ref, "byte terms adc")
    gi, gd = gi.cpu().numpy(), gd.cpu().numpy()
    for j in range(prob.Q):
        assert_topk_matches(gi[j], gd[j], ref[j], np.arange(prob.N), k, "byte terms q%d" % j)
    # the device builder takes no payload
    dev = etf.Context(device=0, stream=torch.cuda.current_stream().cuda_stream)
    dev.pq_set_codebooks(prob.cb)
    dev.index_set_leaf_term(prob.term)
    with pytest.raises(etf.EtfError) as e:
        dev.index_build_device(torch.from_numpy(prob.codes).cuda(), T=2)
    assert e.value.code == -2
