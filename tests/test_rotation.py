"""Rotation in front of the quantiser (Optimized Product Quantization as a preprocessing option): pins of the oracle's
rotate, the library's host functions against it, properties of the OPQ training, and (marked gpu) the device rotation and
an end-to-end search on rotated vectors."""
import numpy as np
import pytest

import oracle
import paper_1509_05186_amd as etf
from parity import assert_topk_matches


def say(*a):
    print(*a, flush=True)


def random_orthogonal(d, seed):
    q, r = np.linalg.qr(np.random.default_rng(seed).standard_normal((d, d)))
    return (q * np.sign(np.diag(r))).astype(np.float32)


# ---- the oracle's rotate, pinned to what mathematics fixes -------------------------------------------------------
def test_oracle_rotate_hand_example_identity_and_permutation():
    # a quarter turn in the plane: (x0, x1) -> (-x1, x0); worked by hand
    R = np.array([[0, -1], [1, 0]], dtype=np.float32)
    x = np.array([[3, 4], [-1.5, 0.25], [0, 0]], dtype=np.float32)
    assert np.array_equal(oracle.rotate(x, R), np.array([[-4, 3], [-0.25, -1.5], [0, 0]], dtype=np.float32))
    # a matrix with one non-trivial row, by hand: y0 = 2 x0 + 0.5 x1 - x2 = 2*1 + 0.5*4 - 3 = 1
    R3 = np.array([[2, 0.5, -1], [0, 1, 0], [0, 0, 1]], dtype=np.float32)
    assert np.array_equal(oracle.rotate(np.array([[1, 4, 3]], dtype=np.float32), R3), np.array([[1, 4, 3]], dtype=np.float32))
    rng = np.random.default_rng(1)
    x = rng.standard_normal((50, 7)).astype(np.float32)
    assert np.array_equal(oracle.rotate(x, np.eye(7, dtype=np.float32)), x)
    perm = rng.permutation(7)
    P = np.zeros((7, 7), dtype=np.float32)
    P[np.arange(7), perm] = 1                                    # y[i] = x[perm[i]]: exact, whatever the order of additions
    assert np.array_equal(oracle.rotate(x, P), x[:, perm])
    # a transposed operand would send x to x[inverse permutation]
    assert not np.array_equal(oracle.rotate(x, P.T), x[:, perm])


def test_oracle_rotate_against_a_library_product_and_norms():
    rng = np.random.default_rng(2)
    d = 48
    x = (rng.standard_normal((200, d)) * 3).astype(np.float32)
    R = random_orthogonal(d, 3)
    y = oracle.rotate(x, R)
    ref = x.astype(np.float64) @ R.astype(np.float64).T          # the definition through a library routine, float64
    assert y.dtype == np.float32
    assert np.all(np.abs(y - ref) <= np.spacing(np.abs(ref).astype(np.float32)) * 0.5 + 1e-12)   # correctly rounded up to the sum's own rounding
    # an orthogonal matrix keeps lengths and distances
    assert np.allclose(np.linalg.norm(y.astype(np.float64), axis=1), np.linalg.norm(x.astype(np.float64), axis=1), rtol=1e-6)
    # order of the additions: ascending dimensions, one rounded addition each (cancellation makes other orders visible)
    big = np.array([[1e8, 1.0, -1e8, 1.0]], dtype=np.float32)
    ones = np.zeros((4, 4), dtype=np.float32)
    ones[0] = 1
    assert oracle.rotate(big, ones)[0, 0] == np.float32(((1e8 + 1.0) - 1e8) + 1.0)   # float64 holds 1e8 + 1 exactly: 2.0
    tiny = np.array([[1e17, 1.0, -1e17, 1.0]], dtype=np.float32)
    a = np.float64(np.float32(1e17))
    assert oracle.rotate(tiny, ones)[0, 0] == np.float32(((a + 1.0) - a) + 1.0)      # 1.0: the first 1 is lost, the second is not


# ---- the library's host side ------------------------------------------------------------------------------------
def test_host_rotate_equals_oracle_and_state():
    rng = np.random.default_rng(4)
    d = 40
    x = (rng.standard_normal((3000, d)) * 2).astype(np.float32)
    R = random_orthogonal(d, 5)
    c = etf.Context(device=None)
    with pytest.raises(etf.EtfError):
        c.pq_get_rotation()
    c.pq_set_rotation(R)
    assert np.array_equal(c.pq_get_rotation(), R)
    assert np.array_equal(c.rotate(x), oracle.rotate(x, R))
    assert c.rotate(x[:0]).shape == (0, d)
    bad = R.copy()
    bad[3, 3] = np.nan
    with pytest.raises(etf.EtfError):
        c.pq_set_rotation(bad)
    c.pq_set_rotation(None)
    with pytest.raises(etf.EtfError):
        c._ck(c._lib.etf_rotate(c._h, x.ctypes.data, 10, x.ctypes.data))


def planted(n, d, M, seed):
    """Vectors whose dimension groups are independent in a hidden basis: tight clusters per group, then a rotation mixes
    the groups.  A product quantiser in the given basis wastes its codewords; in the hidden basis it is nearly lossless."""
    rng = np.random.default_rng(seed)
    ds = d // M
    centres = rng.standard_normal((M, 16, ds)) * 4
    pick = rng.integers(0, 16, size=(n, M))
    z = np.concatenate([centres[m, pick[:, m]] for m in range(M)], axis=1) + rng.standard_normal((n, d)) * 0.05
    Q = random_orthogonal(d, seed + 1).astype(np.float64)
    return (z @ Q.T).astype(np.float32)


def distortion(c, x):
    y = c.rotate(x)
    rec = oracle.decode(c.pq_encode(y), c.pq_get_codebooks())
    return float(np.mean(np.sum((y.astype(np.float64) - rec) ** 2, axis=1)))


def test_opq_train_lowers_the_distortion_and_keeps_the_rotation_orthogonal():
    d, M, K = 16, 4, 16
    x = planted(6000, d, M, 7)
    c = etf.Context(device=None)
    c.opq_train(x, M, K, iters=6, rounds=0, seed=3)              # no round: the product quantiser behind the identity
    assert np.array_equal(c.pq_get_rotation(), np.eye(d, dtype=np.float32))
    plain = distortion(c, x)
    p = etf.Context(device=None)
    p.pq_train(x, M, K, 6, 3)
    assert np.array_equal(p.pq_get_codebooks(), c.pq_get_codebooks())
    c.opq_train(x, M, K, iters=6, rounds=12, seed=3)             # continues from the rotation that is set
    R = c.pq_get_rotation().astype(np.float64)
    assert np.allclose(R @ R.T, np.eye(d), atol=1e-5)
    rotated = distortion(c, x)
    say("  distortion: plain %.3f, after 12 rounds %.3f" % (plain, rotated))
    assert rotated < 0.8 * plain                               # the alternation stops in a local optimum, well below the start
    # codes of rotated vectors by the library are the oracle's for the oracle's rotation
    y = oracle.rotate(x[:500], c.pq_get_rotation())
    assert np.array_equal(c.pq_encode(c.rotate(x[:500])), oracle.encode_f32(y, c.pq_get_codebooks()))


# ---- device -----------------------------------------------------------------------------------------------------
@pytest.mark.gpu
@pytest.mark.parametrize("d,n", [(128, 5000), (96, 1025), (7, 300), (960, 70), (1, 10)])
def test_rotate_device_equals_oracle(d, n):
    torch = pytest.importorskip("torch")
    say("device rotation d", d, "n", n)
    rng = np.random.default_rng(d + n)
    x = (rng.standard_normal((n, d)) * 3).astype(np.float32)
    R = random_orthogonal(d, d) if d > 1 else np.array([[-1.5]], dtype=np.float32)
    c = etf.Context(device=0, stream=torch.cuda.current_stream().cuda_stream)
    c.pq_set_rotation(R)
    y = c.rotate_device(torch.from_numpy(x).cuda())
    torch.cuda.synchronize()
    assert np.array_equal(y.cpu().numpy(), oracle.rotate(x, R))
    assert c.rotate_device(torch.empty((0, d), dtype=torch.float32, device="cuda")).shape == (0, d)
    xd = torch.from_numpy(x).cuda()
    with pytest.raises(etf.EtfError):
        c.rotate_device(xd, out=xd)                              # not in place
    c.pq_set_rotation(None)
    with pytest.raises(etf.EtfError):
        c.rotate_workspace_bytes()


@pytest.mark.gpu
def test_search_behind_a_trained_rotation():
    """OPQ end to end: rotation and codebooks trained by the library, database and queries rotated on the device, the
    rest of the path as ever.  The oracle gets the same rotation and codebooks and does everything itself."""
    torch = pytest.importorskip("torch")
    say("search behind a trained rotation")
    d, M, K, N, Q, k = 32, 8, 64, 20000, 150, 20
    x = planted(N + 4000 + Q, d, M, 11)
    xt, xb, q = x[:4000], x[4000:4000 + N], x[4000 + N:]
    c = etf.Context(device=0, stream=torch.cuda.current_stream().cuda_stream)
    c.opq_train(xt, M, K, iters=5, rounds=4, seed=2)
    R, cb = c.pq_get_rotation(), c.pq_get_codebooks()
    yb = c.rotate_device(torch.from_numpy(xb).cuda())
    codes = c.pq_encode_device(yb)
    torch.cuda.synchronize()
    ref_codes = oracle.encode_f32(oracle.rotate(xb, R), cb)
    assert np.array_equal(codes.cpu().numpy(), ref_codes)
    c.index_build_device(codes, T=2)
    ids, dist = c.search(c.rotate_device(torch.from_numpy(q).cuda()), k, etf.ETF_MODE_FOREST)
    torch.cuda.synchronize()
    ref = oracle.adc_all(oracle.rotate(q, R), cb, ref_codes)
    ids, dist = ids.cpu().numpy(), dist.cpu().numpy()
    for j in range(Q):
        assert_topk_matches(ids[j], dist[j], ref[j], np.arange(N), k, "rotated q%d" % j)
    # an orthogonal rotation keeps the geometry: the same numbers are distances to the reconstructions turned back
    back = oracle.decode(ref_codes[:200], cb) @ R.astype(np.float64)
    direct = ((q[:5, None, :].astype(np.float64) - back[None, :, :]) ** 2).sum(axis=2)
    assert np.allclose(direct, ref[:5, :200], rtol=1e-4)
