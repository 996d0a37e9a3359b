"""GPU parity of the device encoder: codes bit-identical to the float32 assignment of the oracle."""
import numpy as np
import pytest

import oracle
from workload import GaussianMixture, get_config, near_tie_vectors, SEED_DATABASE, SEED_TRAIN

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import paper_1509_05186_amd as etf  # noqa: E402


def say(*a):
    print(*a, flush=True)


KERNELS = [0, 1]     # option encode_kernel: 0 distance evaluations on the matrix cores, 1 the float32 rule throughout


def make(d, M, K, ntrain, seed, iters=3, kernel=0):
    gm = GaussianMixture(d, 8, 1.1, (0.2, 1.0), (-4.0, 4.0), seed=seed)
    xt = gm.sample(ntrain, 1)
    cb, _ = oracle.kmeans(xt, M, K, iters, oracle.kmeans_init_rows(ntrain, M, K, seed))
    c = etf.Context(device=0, stream=torch.cuda.current_stream().cuda_stream)
    c.set_option("encode_kernel", kernel)
    c.pq_set_codebooks(cb)
    return gm, cb, c


@pytest.mark.parametrize("d,M,K,n", [
    (128, 8, 256, 5000),     # 16 dimensions per group (the benchmark's shape), several blocks and a ragged tail
    (240, 2, 256, 700),      # 120 dimensions per group: wide groups, both operands through LDS, last stage short
    (200, 2, 100, 300),      # 100 per group, 100 codewords: rows of the codeword tile beyond the codebook
    (96, 8, 256, 1025),      # 12 per group: padded to 16
    (119, 7, 50, 513),       # 17 per group (odd: unaligned rows), K not a power of two
    (128, 16, 256, 300),     # 8 per group, 16 groups
    (8, 2, 3, 1),            # a single vector, three codewords
])
@pytest.mark.parametrize("kernel", KERNELS)
def test_encode_device_equals_float32_oracle(d, M, K, n, kernel):
    say("device encoder d", d, "M", M, "K", K, "n", n, "kernel", kernel)
    gm, cb, c = make(d, M, K, max(4 * K, 600), seed=d + M, kernel=kernel)
    x = gm.sample(n, 2)
    got = c.pq_encode_device(torch.from_numpy(x).cuda())
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy(), oracle.encode_f32(x, cb))


def test_encode_device_wide_groups_on_the_matrix_cores():
    say("device encoder, 240 dimensions per group (beyond the plain kernel's registers)")
    gm, cb, c = make(480, 2, 256, 1200, seed=5)
    x = gm.sample(3000, 2)
    got = c.pq_encode_device(torch.from_numpy(x).cuda())
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy(), oracle.encode_f32(x, cb))
    c.set_option("encode_wide", 0)                       # the general matrix-core kernel on the same input
    again = c.pq_encode_device(torch.from_numpy(x).cuda())
    torch.cuda.synchronize()
    assert torch.equal(again, got)
    c.set_option("encode_kernel", 1)
    with pytest.raises(etf.EtfError):
        c.pq_encode_device(torch.from_numpy(x).cuda())


@pytest.mark.parametrize("kernel", KERNELS)
@pytest.mark.parametrize("d,M,K", [(128, 8, 256), (96, 8, 64), (240, 2, 256)])
def test_encode_device_near_ties_follow_the_float32_rule(d, M, K, kernel):
    """Vectors half way between two codewords up to a few units in the last place: the decision depends on the
    rounding of every single operation (a fused multiply-add in the sum decides thousands of them differently, see
    tests/test_oracle_pins.py::test_encode_f32_near_ties_tell_fused_from_unfused)."""
    say("device encoder on near-ties, d", d, "M", M, "K", K, "kernel", kernel)
    gm, cb, c = make(d, M, K, max(4 * K, 600), seed=2 * d + M, kernel=kernel)
    x = near_tie_vectors(cb, 40000, seed=d)
    got = c.pq_encode_device(torch.from_numpy(x).cuda())
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy(), oracle.encode_f32(x, cb))


@pytest.mark.parametrize("kernel", KERNELS)
def test_encode_device_exact_ties_and_duplicates(kernel):
    say("device encoder: identical codewords and vectors equal to codewords, kernel", kernel)
    cb = np.zeros((2, 8, 4), dtype=np.float32)
    rng = np.random.default_rng(3)
    cb[:, :4] = rng.normal(size=(2, 4, 4)).astype(np.float32)
    cb[:, 4:] = cb[:, :4]                      # every codeword exists twice: the lower index must win
    c = etf.Context(device=0, stream=torch.cuda.current_stream().cuda_stream)
    c.set_option("encode_kernel", kernel)
    c.pq_set_codebooks(cb)
    x = np.concatenate([np.concatenate([cb[0, i % 4], cb[1, (i + 1) % 4]])[None] for i in range(70)]).astype(np.float32)
    got = c.pq_encode_device(torch.from_numpy(x).cuda()).cpu().numpy()
    assert got.max() < 4
    assert np.array_equal(got, oracle.encode_f32(x, cb))


def test_encode_device_one_chunk_of_the_benchmark_database():
    cfg = get_config("cfg2")
    say("device encoder: the first 131072 vectors of cfg2's database against cfg2's library-trained codebooks")
    gm = GaussianMixture.from_config(cfg)
    host = etf.Context(device=None)
    host.pq_train(gm.sample(cfg.n_train, SEED_TRAIN), cfg.M, cfg.K, cfg.kmeans_iters, seed=SEED_TRAIN)
    cb = host.pq_get_codebooks()
    c = etf.Context(device=0, stream=torch.cuda.current_stream().cuda_stream)
    c.pq_set_codebooks(cb)
    x = next(iter(gm.chunks(1 << 17, SEED_DATABASE)))
    got = c.pq_encode_device(torch.from_numpy(x).cuda()).cpu().numpy()
    assert np.array_equal(got, oracle.encode_f32(x, cb))
    # and the host encoder of the library takes the same float32 decisions
    assert np.array_equal(got, host.pq_encode(x))


def test_encode_device_empty_and_errors():
    say("device encoder: n = 0, too many dimensions per group, small workspace")
    _, cb, c = make(16, 2, 4, 100, seed=9)
    out = c.pq_encode_device(torch.empty((0, 16), dtype=torch.float32, device="cuda"))
    assert out.shape == (0, 2)
    with pytest.raises(etf.EtfError):
        c.pq_encode_device(torch.zeros((4, 16), dtype=torch.float32, device="cuda"),
                           ws=torch.empty(64, dtype=torch.uint8, device="cuda"))
    big = np.zeros((1, 2, 130), dtype=np.float32)
    big[0, 1] = 1
    c2 = etf.Context(device=0, stream=torch.cuda.current_stream().cuda_stream)
    c2.set_option("encode_kernel", 1)
    c2.pq_set_codebooks(big)
    with pytest.raises(etf.EtfError):
        c2.pq_encode_device(torch.zeros((4, 130), dtype=torch.float32, device="cuda"))
