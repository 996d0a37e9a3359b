"""The probe kernels behind the benchmark's ceilings (etf_probe_bandwidth): every kind runs on small buffers, the
ones that move data move the right data, the ones that only measure leave the buffers alone, bad arguments are
refused."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import paper_1509_05186_amd as etf  # noqa: E402


def say(*a):
    print(*a, flush=True)


@pytest.fixture(scope="module")
def ctx():
    return etf.Context(device=0, stream=torch.cuda.current_stream().cuda_stream)


@pytest.mark.parametrize("nbytes", [1 << 16, (1 << 20) + 256 * 37])      # the smallest size; a ragged number of rows
def test_streaming_probes_move_the_right_bytes(ctx, nbytes):
    say("probe kernels: copy / write / read / rows on", nbytes, "bytes")
    g = torch.Generator(device="cuda").manual_seed(7)
    a = torch.randint(0, 256, (nbytes,), dtype=torch.uint8, device="cuda", generator=g)
    b = torch.zeros(max(nbytes, 1 << 14), dtype=torch.uint8, device="cuda")
    a0 = a.clone()
    ctx.probe_bandwidth(etf.ETF_PROBE_COPY, a, b, nbytes)
    torch.cuda.synchronize()
    assert torch.equal(b[:nbytes], a0) and torch.equal(a, a0)
    for kind in (etf.ETF_PROBE_READ, etf.ETF_PROBE_ROWS):                 # readers: a is untouched, b gets a word per workgroup
        ctx.probe_bandwidth(kind, a, b, nbytes)
        torch.cuda.synchronize()
        assert torch.equal(a, a0)
    ctx.probe_bandwidth(etf.ETF_PROBE_WRITE, a, b, nbytes)
    torch.cuda.synchronize()
    words = a.view(torch.int32).cpu().numpy().reshape(-1, 4)
    assert np.array_equal(words, np.tile(np.array([1, 2, 3, 4], dtype=np.int32), (nbytes // 16, 1)))


def test_on_chip_probes_run_and_touch_nothing_else(ctx):
    say("probe kernels: LDS reads, vector issue, matrix instruction")
    a = torch.full((1 << 16,), 5, dtype=torch.uint8, device="cuda")
    b = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")
    for kind, amount in ((etf.ETF_PROBE_LDS, 1 << 30), (etf.ETF_PROBE_LDS_SCATTER, 1 << 30),
                         (etf.ETF_PROBE_VALU_F32, 2048 * 256 * 64 * 8), (etf.ETF_PROBE_VALU_ADD3, 2048 * 256 * 64 * 8),
                         (etf.ETF_PROBE_VALU_PK16, 2048 * 256 * 64 * 8), (etf.ETF_PROBE_MFMA_F32, 2048 * 4 * 32 * 4096 * 4)):
        ctx.probe_bandwidth(kind, a, b, amount)
        torch.cuda.synchronize()
        assert int(a.min()) == 5 and int(a.max()) == 5                    # `a` is not used by these kinds


def test_probe_errors(ctx):
    say("probe kernels: refused arguments")
    a = torch.zeros((1 << 16) + 256, dtype=torch.uint8, device="cuda")
    b = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")
    with pytest.raises(etf.EtfError):
        ctx.probe_bandwidth(99, a, b, 1 << 16)                             # unknown kind
    with pytest.raises(etf.EtfError):
        ctx.probe_bandwidth(etf.ETF_PROBE_READ, a, b, 1 << 12)             # too small
    with pytest.raises(etf.EtfError):
        ctx.probe_bandwidth(etf.ETF_PROBE_READ, a, b, (1 << 16) + 8)       # not a multiple of 256
    with pytest.raises(etf.EtfError):
        ctx.probe_bandwidth(etf.ETF_PROBE_READ, a[8:], b, 1 << 16)         # not aligned
    host = etf.Context(device=None)
    with pytest.raises(etf.EtfError):
        host.probe_bandwidth(etf.ETF_PROBE_READ, a, b, 1 << 16)
