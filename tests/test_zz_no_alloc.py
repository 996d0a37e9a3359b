"""The allocation-free search entry point (etf_search_static) against etf_search, through the C ABI: two calls in a
row on one context, the second with fewer queries, each bit for bit what etf_search returns for the same input.
Runs last (file name), alone or after the other tests."""
import numpy as np
import pytest

import oracle
from workload import GaussianMixture
from parity import assert_topk_matches

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import paper_1509_05186_amd as etf  # noqa: E402


def say(*a):
    print(*a, flush=True)


def test_search_static_equals_search_on_two_calls_in_a_row():
    gm = GaussianMixture(32, 16, 1.1, (0.2, 1.0), (-4.0, 4.0), seed=21)
    xt, xb, q = gm.sample(4000, 1), gm.sample(60000, 2), gm.sample(700, 3)
    M, K, k = 8, 256, 50
    cb, _ = oracle.kmeans(xt, M, K, 3, oracle.kmeans_init_rows(4000, M, K, 21))
    codes = oracle.encode(xb, cb)
    c = etf.Context(device=0, stream=torch.cuda.current_stream().cuda_stream)
    c.pq_set_codebooks(cb)
    c.index_build(codes, T=2)
    c.index_upload()
    lib = etf.load_library()
    assert lib.etf_static_scratch_bytes() == 64 << 20
    for nq in (700, 130):            # several batches of tiles with a ragged last tile; then a smaller input
        say("etf_search_static, Q =", nq)
        qd = torch.from_numpy(q[:nq]).cuda()
        want_i, want_d = c.search(qd, k, etf.ETF_MODE_FOREST)
        torch.cuda.synchronize()
        got_i = torch.full((nq, k), -7, dtype=torch.int32, device="cuda")
        got_d = torch.full((nq, k), -7.0, dtype=torch.float32, device="cuda")
        c.search_static(qd, k, etf.ETF_MODE_FOREST, got_i, got_d)
        torch.cuda.synchronize()
        assert torch.equal(got_i, want_i) and torch.equal(got_d, want_d)
        assert c.last_fallback_count() == 0
        ref = oracle.adc_all(q[:4], cb, codes)
        for j in range(4):
            assert_topk_matches(got_i[j].cpu().numpy(), got_d[j].cpu().numpy(), ref[j], np.arange(len(codes)), k, "static q%d" % j)
    # the single tree through the same entry point, and a request that cannot fit the fixed scratch
    t = etf.Context(device=0, stream=torch.cuda.current_stream().cuda_stream)
    t.pq_set_codebooks(cb)
    t.index_build(codes, T=1)
    t.index_upload()
    qd = torch.from_numpy(q[:70]).cuda()
    want = t.search(qd, k, etf.ETF_MODE_TREE)
    got_i = torch.empty((70, k), dtype=torch.int32, device="cuda")
    got_d = torch.empty((70, k), dtype=torch.float32, device="cuda")
    t.search_static(qd, k, etf.ETF_MODE_TREE, got_i, got_d)
    torch.cuda.synchronize()
    assert torch.equal(got_i, want[0]) and torch.equal(got_d, want[1])
    t.set_option("cand_cap", 1 << 18)       # 64 queries x 2^18 candidates x 8 bytes = 128 MiB for one tile
    with pytest.raises(etf.EtfError) as e:
        t.search_static(qd, k, etf.ETF_MODE_TREE, got_i, got_d)
    assert e.value.code == -3 and "scratch" in str(e.value)
