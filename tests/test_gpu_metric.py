"""GPU parity of the scalar-product payload (option metric = 1): tables, all-pairs sums and searches for the largest
products against the float64 oracle, on the same indexes and kernels as the distance searches."""
import numpy as np
import pytest

import oracle
from parity import ip_scale, assert_topk_ip_matches
from test_gpu_parity import Problem, qdev, say, FLAT, TREE, FOREST

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import paper_1509_05186_amd as etf  # noqa: E402

IP_TOL = 1e-5


class IpProblem(Problem):
    @property
    def ref_ip(self):
        if getattr(self, "_ip", None) is None:
            self._ip = oracle.adc_all_ip(self.q, self.cb, self.codes)
            self._scale = np.array([ip_scale(oracle.lut_ip(q, self.cb)) for q in self.q])
        return self._ip

    @property
    def scale(self):
        self.ref_ip
        return self._scale


@pytest.fixture(scope="module")
def small():
    return IpProblem(d=32, M=8, K=256, N=20000, Q=150, ntrain=4000, seed=11)


@pytest.fixture(scope="module")
def dups():
    return IpProblem(d=16, M=4, K=4, N=6000, Q=70, ntrain=500, seed=12, dup_factor=3)


@pytest.mark.parametrize("lut_kernel", [0, 1])     # 0: the contraction on the matrix cores, 1: plain float32 sums
def test_scalar_product_tables(small, lut_kernel):
    say("scalar-product tables, table kernel", lut_kernel)
    p = small
    c = p.ctx(T=1, metric=1, lut_kernel=lut_kernel)
    lut = c.lut_build(qdev(p)).cpu().numpy().astype(np.float64)
    M, K, ds = p.cb.shape
    for j in range(0, p.Q, 7):
        ref = oracle.lut_ip(p.q[j], p.cb)
        mag = np.abs(p.cb.astype(np.float64)) @ np.abs(p.q[j].astype(np.float64)).reshape(M, ds, 1)    # sum |q_i| |c_i|
        assert np.all(np.abs(lut[j] - ref) <= IP_TOL * mag[:, :, 0]), j


def test_scalar_product_tables_odd_group_width():
    say("scalar-product tables: 17 dimensions per group, 50 codewords, a ragged tile of queries")
    p = IpProblem(d=119, M=7, K=50, N=500, Q=70, ntrain=600, seed=21)
    M, K, ds = p.cb.shape
    for lut_kernel in (0, 1):
        c = p.ctx(T=1, metric=1, lut_kernel=lut_kernel)
        lut = c.lut_build(qdev(p)).cpu().numpy().astype(np.float64)
        for j in range(p.Q):
            ref = oracle.lut_ip(p.q[j], p.cb)
            mag = np.abs(p.cb.astype(np.float64)) @ np.abs(p.q[j].astype(np.float64)).reshape(M, ds, 1)
            assert np.all(np.abs(lut[j] - ref) <= IP_TOL * mag[:, :, 0]), (lut_kernel, j)
        got = c.adc(qdev(p), TREE).cpu().numpy().astype(np.float64)
        assert np.all(np.abs(got - p.ref_ip) <= IP_TOL * p.scale[:, None])


@pytest.mark.parametrize("trav", [0, 1, 2])
@pytest.mark.parametrize("mode,T", [(FLAT, 1), (TREE, 1), (FOREST, 2), (FOREST, 4)])
def test_scalar_product_all_pairs(small, mode, T, trav):
    if mode == FLAT and trav == 1:
        pytest.skip("flat mode has no tree traversal")
    say("scalar products, all pairs, mode", mode, "T", T, "traversal", trav)
    p = small
    c = p.ctx(T=T, metric=1, traversal=trav)
    got = c.adc(qdev(p), mode)
    torch.cuda.synchronize()
    err = np.abs(got.cpu().numpy().astype(np.float64) - p.ref_ip)
    assert np.all(err <= IP_TOL * p.scale[:, None]), float((err / p.scale[:, None]).max())


def check_ip_search(p, c, mode, k, ids=None, what=""):
    oi, ov = c.search(qdev(p), k, mode)
    torch.cuda.synchronize()
    oi, ov = oi.cpu().numpy(), ov.cpu().numpy()
    idv = np.arange(p.N) if ids is None else ids
    for j in range(p.Q):
        assert_topk_ip_matches(oi[j], ov[j], p.ref_ip[j], idv, k, IP_TOL * p.scale[j], "%s q%d" % (what, j))
    return oi, ov


@pytest.mark.parametrize("trav", [0, 1, 2])
@pytest.mark.parametrize("mode,T", [(FLAT, 1), (TREE, 1), (FOREST, 2), (FOREST, 4)])
@pytest.mark.parametrize("k", [1, 100])
def test_scalar_product_search(small, mode, T, k, trav):
    if mode == FLAT and trav == 1:
        pytest.skip("flat mode has no tree traversal")
    say("largest scalar products, mode", mode, "T", T, "k", k, "traversal", trav)
    c = small.ctx(T=T, metric=1, sample_min=2048, traversal=trav)
    check_ip_search(small, c, mode, k, what="ip m%d T%d k%d" % (mode, T, k))
    assert c.last_fallback_count() == 0


@pytest.mark.parametrize("mode,T", [(FLAT, 1), (FOREST, 2)])
def test_scalar_product_search_exact_kernel_and_ties(dups, mode, T):
    say("largest scalar products with repeated encodings and explicit ids; the exact kernel; mode", mode)
    p = dups
    ids = np.random.default_rng(5).permutation(3 * p.N)[: p.N].astype(np.int32)
    c = p.ctx(T=T, ids=ids, metric=1)
    a = check_ip_search(p, c, mode, 50, ids, "ip dups")
    c.set_option("force_fallback", 1)
    b = check_ip_search(p, c, mode, 50, ids, "ip dups exact kernel")
    assert c.last_fallback_count() == p.Q
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_metric_switches_per_call_and_matches_oracle_search(small):
    say("one index, both metrics in turn; lists equal to the oracle's where it has no near-ties")
    p = small
    c = p.ctx(T=2)
    d0 = c.search(qdev(p), 10, FOREST)
    c.set_option("metric", 1)
    oi, ov = c.search(qdev(p), 10, FOREST)
    c.set_option("metric", 0)
    d1 = c.search(qdev(p), 10, FOREST)
    torch.cuda.synchronize()
    assert torch.equal(d0[0], d1[0]) and torch.equal(d0[1], d1[1])
    ri, rv = oracle.search_ip(p.q, p.cb, p.codes, 10)
    assert (oi.cpu().numpy() == ri).mean() > 0.99
    assert np.all(np.abs(ov.cpu().numpy() - rv) <= IP_TOL * p.scale[:, None])
    with pytest.raises(etf.EtfError):
        c.set_option("metric", 2)


@pytest.mark.parametrize("N,Q,k", [(50, 5, 10), (1, 3, 1), (300, 130, 300)])
def test_scalar_product_search_tiny_databases(N, Q, k):
    say("largest scalar products on a tiny database: every encoding is a candidate; N", N, "Q", Q, "k", k)
    p = IpProblem(d=16, M=4, K=16, N=N, Q=Q, ntrain=200, seed=31)
    for mode, T in [(FLAT, 1), (TREE, 1), (FOREST, 2)]:
        c = p.ctx(T=T, metric=1)
        check_ip_search(p, c, mode, k, what="ip tiny m%d" % mode)


def test_scalar_product_search_several_batches_and_device_built_index(small):
    say("largest scalar products: a workspace cap that forces several query batches; a device-built index")
    p = small
    c = p.ctx(T=2, metric=1, sample_min=2048, ws_cap_bytes=8 << 20)
    a = check_ip_search(p, c, FOREST, 10, what="ip batched")
    d = etf.Context(device=0, stream=torch.cuda.current_stream().cuda_stream)
    d.set_option("metric", 1)
    d.set_option("sample_min", 2048)
    d.pq_set_codebooks(p.cb)
    d.index_build_device(torch.from_numpy(p.codes).cuda(), T=2)
    b = check_ip_search(p, d, FOREST, 10, what="ip device-built")
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
