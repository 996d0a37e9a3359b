"""A search is plain stream work (kernels only, no allocation, no memset, no synchronisation), so it can be
captured into a HIP graph and replayed."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import paper_1509_05186_amd as etf  # noqa: E402
from test_gpu_parity import Problem, say  # noqa: E402


@pytest.mark.parametrize("mode,T,trav", [(etf.ETF_MODE_FOREST, 2, 2), (etf.ETF_MODE_FOREST, 2, 0), (etf.ETF_MODE_FLAT, 1, 2)])
def test_search_captured_in_a_graph_replays_identically(mode, T, trav):
    say("graph capture of etf_search, mode", mode, "T", T, "traversal", trav)
    p = Problem(d=32, M=8, K=256, N=20000, Q=150, ntrain=4000, seed=11)
    c = p.ctx(T=T, sample_min=2048, traversal=trav)
    qd = torch.from_numpy(p.q).cuda()
    k = 20
    ws = c.alloc_workspace(p.Q, k, mode)
    want_i, want_d = c.search(qd, k, mode, ws=ws)
    torch.cuda.synchronize()
    want_i, want_d = want_i.clone(), want_d.clone()
    out_i = torch.zeros((p.Q, k), dtype=torch.int32, device="cuda")
    out_d = torch.zeros((p.Q, k), dtype=torch.float32, device="cuda")
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        c.set_stream(torch.cuda.current_stream().cuda_stream)      # the capturing stream
        c.search(qd, k, mode, out_i, out_d, ws)
    c.set_stream(torch.cuda.current_stream().cuda_stream)
    for r in range(3):
        out_i.fill_(-1)
        out_d.fill_(-1.0)
        # eager work of the program between the replays, on the same workspace
        other_i, other_d = c.search(qd.flip(0).contiguous(), k, mode, ws=ws)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out_i, want_i) and torch.equal(out_d, want_d), "replay %d differs from the eager result" % r
        assert torch.equal(other_i.flip(0), want_i)
