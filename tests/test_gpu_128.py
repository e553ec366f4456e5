"""GPU-vs-oracle parity of the Z_2^128 entry points (Section 6: 64-bit or 128-bit rings): share, open,
elementwise Beaver mul, truncation, and the Beaver matmul on both GEMM paths, bit for bit."""
import numpy as np
import pytest
import torch

import oracle
from oracle import r128
from paper_2402_02320_amd import spin

pytestmark = pytest.mark.gpu
R = spin.ring128


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int64)).cuda()


def host(t):
    return t.cpu().numpy().view(np.uint64)


def rand_ring(rng, shape):
    return rng.integers(0, 1 << 64, size=tuple(shape) + (2,), dtype=np.uint64)


@pytest.mark.parametrize("n", [1, 2, 3, 5, 8])
@pytest.mark.parametrize("count", [1, 2, 777, 40001])
def test_share_open_mul_trunc(n, count):
    rng = np.random.default_rng(n * 1000 + count)
    x, y = rand_ring(rng, (count,)), rand_ring(rng, (count,))
    xs, ys = r128.share(x, n, 7, 1), r128.share(y, n, 7, 2)
    xd = R.share(dev(x), n, 7, 1)
    assert (host(xd) == xs).all()
    assert (host(R.open(xd)) == x).all()
    m = rand_ring(rng, (n, count))
    assert (host(R.open(xd, dev(m))) == r128.open_(xs, m)).all()
    a, b, c = r128.dealer_mul(n, count, seed=7)
    want = r128.beaver_mul(xs, ys, a, b, c)
    zd = R.beaver_mul(xd, dev(ys), dev(a), dev(b), dev(c))
    assert (host(zd) == want).all()
    for f in (1, 16, 40, 125):
        r, rt, rm = r128.trunc_dealer(n, count, f, seed=9 + f)
        # any share values exercise the combine; the closed form is pinned on the oracle side
        assert (host(R.trunc(zd, dev(r), dev(rt), dev(rm), f)) == r128.trunc(want, r, rt, rm, f)).all()


PATHS = [pytest.param(spin.LIMB_MFMA, id="limb"), pytest.param(spin.VALU, id="valu")]
SHAPES = [(1, 1, 1, 1, 1), (2, 1, 33, 31, 32), (3, 2, 70, 65, 45), (5, 1, 64, 64, 64), (8, 1, 40, 40, 40),
          (2, 3, 17, 130, 100), (3, 1, 129, 200, 257)]


@pytest.mark.parametrize("path", PATHS)
@pytest.mark.parametrize("n,batch,M,N,K", SHAPES)
def test_beaver_matmul(n, batch, M, N, K, path):
    rng = np.random.default_rng(n * 7 + M)
    X, Y = rand_ring(rng, (n, batch, M, K)), rand_ring(rng, (n, batch, K, N))
    A, B, C = r128.dealer_matmul(n, batch, M, N, K, seed=n * 7 + M)
    want = r128.beaver_matmul(X, Y, A, B, C)
    got = R.beaver_matmul(dev(X), dev(Y), dev(A), dev(B), dev(C), path=path)
    assert (host(got) == want).all()
    # reconstruction against the plain definition
    z = r128.open_(want)
    x, y = r128.open_(X), r128.open_(Y)
    for b in range(batch):
        assert (z[b] == r128.ring_matmul(x[b], y[b])).all()


def test_limb_path_worst_case_digits_across_the_inner_dimension_split():
    # all sixteen digits of every operand equal to -128 (value 0x7F..7F80), K beyond one accumulation chunk
    n, M, N, K = 2, 32, 32, 170 * 32 + 64
    worst = np.array([0x7F7F7F7F7F7F7F80, 0x7F7F7F7F7F7F7F7F], dtype=np.uint64)
    X = np.zeros((n, 1, M, K, 2), dtype=np.uint64); Y = np.zeros((n, 1, K, N, 2), dtype=np.uint64)
    A = np.zeros_like(X); B = np.zeros_like(Y)
    X[0] = worst; X[1] = worst; Y[0] = worst; Y[1] = worst; A[1] = worst; B[1] = worst     # E = F = A_1 = B_1 = worst
    C = np.zeros((n, 1, M, N, 2), dtype=np.uint64)
    want = r128.beaver_matmul(X, Y, A, B, C)
    got = R.beaver_matmul(dev(X), dev(Y), dev(A), dev(B), dev(C), path=spin.LIMB_MFMA)
    assert (host(got) == want).all()


@pytest.mark.parametrize("path", PATHS)
def test_matmul_1024_cube_two_parties(path):
    # config 2's GEMM shape on the 128-bit ring
    rng = np.random.default_rng(2)
    n, M = 2, 1024
    X, Y = rand_ring(rng, (n, 1, M, M)), rand_ring(rng, (n, 1, M, M))
    A, B, C = rand_ring(rng, (n, 1, M, M)), rand_ring(rng, (n, 1, M, M)), rand_ring(rng, (n, 1, M, M))
    rows = slice(0, 1024, 37)
    want = r128.beaver_matmul(X[:, :, rows], Y, A[:, :, rows], B, C[:, :, rows])      # rows of Z depend on rows of X, A, C only
    got = R.beaver_matmul(dev(X), dev(Y), dev(A), dev(B), dev(C), path=path)
    assert (host(got)[:, :, rows] == want).all()


def test_streaming_sizes():
    # past 64 MB per call the elementwise kernels use their non-temporal variants
    n, count, f = 3, (1 << 21) + 1, 40
    rng = np.random.default_rng(128)
    x, y = rand_ring(rng, (count,)), rand_ring(rng, (count,))
    xs, ys = r128.share(x, n, 7, 1), r128.share(y, n, 7, 2)
    xd = R.share(dev(x), n, 7, 1)
    assert (host(xd) == xs).all()
    a, b, c = r128.dealer_mul(n, count, seed=7)
    assert (host(R.open(xd, dev(a))) == r128.open_(xs, a)).all()
    want = r128.beaver_mul(xs, ys, a, b, c)
    zd = R.beaver_mul(xd, dev(ys), dev(a), dev(b), dev(c))
    assert (host(zd) == want).all()
    r, rt, rm = r128.trunc_dealer(n, count, f, seed=9)
    assert (host(R.trunc(zd, dev(r), dev(rt), dev(rm), f)) == r128.trunc(want, r, rt, rm, f)).all()
