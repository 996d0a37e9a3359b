"""Chunk order on the GPU: an index whose encodings hold the chunks in another order gives the same distances and
neighbours (the lookup tables are reordered to match), from the host builder and from the device builder."""
import numpy as np
import pytest

import oracle
from parity import assert_distances_close, ip_scale
from test_gpu_parity import Problem, qdev, say, check_search, FLAT, TREE, FOREST
from test_gpu_build import dev_ctx, check_image, assert_same_as_host_build

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import paper_1509_05186_amd as etf  # noqa: E402

ORDER8 = [5, 2, 7, 0, 1, 6, 3, 4]


@pytest.fixture(scope="module")
def small():
    return Problem(d=32, M=8, K=256, N=20000, Q=150, ntrain=4000, seed=11)


def host_ordered(p, T, order, **opts):
    c = etf.Context(device=0, stream=torch.cuda.current_stream().cuda_stream)
    for name, v in opts.items():
        c.set_option(name, v)
    c.pq_set_codebooks(p.cb)
    c.index_set_chunk_order(order)
    c.index_build(p.codes, T=T)
    c.index_upload()
    return c


@pytest.mark.parametrize("trav", [0, 1, 2])
@pytest.mark.parametrize("mode,T", [(FLAT, 1), (TREE, 1), (FOREST, 2), (FOREST, 4)])
def test_reordered_index_gives_the_same_answers(small, mode, T, trav):
    if mode == FLAT and trav == 1:
        pytest.skip("flat mode has no tree traversal")
    say("chunk order", ORDER8, "mode", mode, "T", T, "traversal", trav)
    p = small
    c = host_ordered(p, T, ORDER8, sample_min=2048, traversal=trav)
    dist = c.adc(qdev(p), mode)
    torch.cuda.synchronize()
    assert_distances_close(dist.cpu().numpy(), p.ref_all, "all pairs, reordered chunks")
    for k in (1, 100):
        check_search(p, c, mode, k, what="reordered m%d T%d k%d" % (mode, T, k))
    assert c.last_fallback_count() == 0
    # the public tables stay in the quantiser's order
    lut = c.lut_build(qdev(p)[:4]).cpu().numpy()
    for j in range(4):
        assert_distances_close(lut[j], oracle.lut(p.q[j], p.cb), "public tables")


@pytest.mark.parametrize("lut_kernel", [0, 1])
def test_reordered_index_exact_kernel_and_both_table_kernels(small, lut_kernel):
    say("chunk order: exact kernel, table kernel", lut_kernel)
    p = small
    c = host_ordered(p, 2, ORDER8, lut_kernel=lut_kernel, force_fallback=1)
    check_search(p, c, FOREST, 20, what="reordered exact")
    assert c.last_fallback_count() == p.Q


def test_reordered_index_built_on_the_device(small):
    say("chunk order: device build equals host build, searches agree")
    p = small
    c, img = dev_ctx(p.cb, p.codes, None, T=2, order=ORDER8, sample_min=2048)
    assert c.index_stats()["chunk_order"] == ORDER8
    check_image(c, img, p.codes[:, ORDER8], None)
    assert_same_as_host_build(c, img, p.cb, p.codes, None, 2, None, order=ORDER8, sample_min=2048)
    h = host_ordered(p, 2, ORDER8, sample_min=2048)
    a, b = c.search(qdev(p), 50, FOREST), h.search(qdev(p), 50, FOREST)
    torch.cuda.synchronize()
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])
    check_search(p, c, FOREST, 50, what="reordered device-built")
    # sixteen chunks, four trees, a random order
    w = Problem(d=64, M=16, K=256, N=12000, Q=70, ntrain=3000, seed=13)
    order16 = np.random.default_rng(2).permutation(16).tolist()
    c2, img2 = dev_ctx(w.cb, w.codes, None, T=4, order=order16, sample_min=1024)
    assert_same_as_host_build(c2, img2, w.cb, w.codes, None, 4, None, order=order16, sample_min=1024)
    check_search(w, c2, FOREST, 20, what="reordered M16")


def test_reordered_index_scalar_products(small):
    say("chunk order with scalar-product tables")
    p = small
    c = host_ordered(p, 2, ORDER8, metric=1)
    got = c.adc(qdev(p), FOREST).cpu().numpy().astype(np.float64)
    ref = oracle.adc_all_ip(p.q, p.cb, p.codes)
    scale = np.array([ip_scale(oracle.lut_ip(q, p.cb)) for q in p.q])
    assert np.all(np.abs(got - ref) <= 1e-5 * scale[:, None])
    oi, ov = c.search(qdev(p), 10, FOREST)
    ri, rv = oracle.search_ip(p.q, p.cb, p.codes, 10)
    assert (oi.cpu().numpy() == ri).mean() > 0.99 and np.all(np.abs(ov.cpu().numpy() - rv) <= 1e-5 * scale[:, None])


def test_suggested_order_on_structured_codes():
    say("suggested chunk order: fewer lookups, same answers")
    p = Problem(d=32, M=8, K=256, N=20000, Q=70, ntrain=4000, seed=14)
    c = etf.Context(device=0, stream=torch.cuda.current_stream().cuda_stream)
    c.pq_set_codebooks(p.cb)
    order, given, best = c.suggest_chunk_order(p.codes, T=2)
    assert sorted(order.tolist()) == list(range(8)) and best <= given
    c.index_set_chunk_order(order)
    c.index_build(p.codes, T=2)
    c.index_upload()
    assert sum(t["lookups"] for t in c.index_stats()["trees"]) == best
    check_search(p, c, FOREST, 10, what="suggested order")
