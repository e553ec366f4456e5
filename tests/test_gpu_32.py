"""GPU-vs-oracle parity of the Z_2^32 entry points (the Fixed32 representation of Section 7.1): the local
cast from Fixed64, share, open, elementwise Beaver mul, truncation, and the Beaver matmul on both GEMM
paths, bit for bit.  The oracle is the l-parametrised C code at l = 32 (ring elements in uint64 storage)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2402_02320_amd import spin

pytestmark = pytest.mark.gpu
R = spin.ring32
M32 = np.uint64(0xFFFFFFFF)


def dev(a):                      # oracle array (uint64 storage of 32-bit ring elements) -> int32 CUDA tensor
    a = np.asarray(a)
    assert a.max(initial=0) <= M32
    return torch.from_numpy(np.ascontiguousarray(a.astype(np.uint32)).view(np.int32)).cuda()


def dev64(a):
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int64)).cuda()


def host(t):
    return t.cpu().numpy().view(np.uint32).astype(np.uint64)


def rand_ring(rng, shape):
    return rng.integers(0, 1 << 32, size=shape, dtype=np.uint64)


@pytest.mark.parametrize("n", [1, 2, 3, 5, 8])
@pytest.mark.parametrize("count", [1, 2, 3, 4, 778, 1001, 40004])      # odd, 2 mod 4 and 0 mod 4 lane forms
def test_share_open_mul_trunc(n, count):
    rng = np.random.default_rng(n * 1000 + count)
    x, y = rand_ring(rng, count), rand_ring(rng, count)
    xs, ys = oracle.share(x, n, 7, 1, l=32), oracle.share(y, n, 7, 2, l=32)
    xd = R.share(dev(x), n, 7, 1)
    assert (host(xd) == xs).all()
    assert (host(R.open(xd)) == x).all()
    m = rand_ring(rng, (n, count))
    assert (host(R.open(xd, dev(m))) == oracle.open_(xs, m, l=32)).all()
    a, b, c = oracle.dealer_mul(n, count, seed=7, l=32)
    want = oracle.beaver_mul(xs, ys, a, b, c, l=32)
    zd = R.beaver_mul(xd, dev(ys), dev(a), dev(b), dev(c))
    assert (host(zd) == want).all()
    for f in (1, 8, 16, 29):
        r, rt, rm = oracle.trunc_dealer(n, count, f, seed=9 + f, l=32)
        # any share values exercise the combine; the closed form is pinned on the oracle side
        assert (host(R.trunc(zd, dev(r), dev(rt), dev(rm), f)) == oracle.trunc(want, r, rt, rm, f, l=32)).all()
    # in place
    R.beaver_mul(xd, dev(ys), dev(a), dev(b), dev(c), out=xd)
    assert (host(xd) == want).all()


def test_streaming_sizes():
    # past 64 MB per call the kernels use their non-temporal variants
    n, count = 5, (1 << 22) + 2
    rng = np.random.default_rng(5)
    x, y = rand_ring(rng, count), rand_ring(rng, count)
    xs, ys = oracle.share(x, n, 3, 1, l=32), oracle.share(y, n, 3, 2, l=32)
    a, b, c = oracle.dealer_mul(n, count, seed=4, l=32)
    r, rt, rm = oracle.trunc_dealer(n, count, 8, seed=5, l=32)
    xd = R.share(dev(x), n, 3, 1)
    assert (host(xd) == xs).all()
    assert (host(R.open(xd, dev(a))) == oracle.open_(xs, a, l=32)).all()
    zo = oracle.beaver_mul(xs, ys, a, b, c, l=32)
    zd = R.beaver_mul(xd, dev(ys), dev(a), dev(b), dev(c))
    assert (host(zd) == zo).all()
    assert (host(R.trunc(zd, dev(r), dev(rt), dev(rm), 8)) == oracle.trunc(zo, r, rt, rm, 8, l=32)).all()


@pytest.mark.parametrize("count", [1, 2, 999, 1 << 16, (1 << 23) + 2])
def test_cast_from_fixed64(count):
    rng = np.random.default_rng(count)
    n = 3
    x = rng.integers(-(1 << 31), 1 << 31, size=count, dtype=np.int64)
    X64 = oracle.share(x.view(np.uint64), n, 50, oracle.STREAM_X)
    got = R.cast_from_64(dev64(X64))
    assert (host(got) == oracle.cast_64_to_32(X64)).all()
    assert (host(R.open(got)) == x.view(np.uint64) & M32).all()


PATHS = [pytest.param(spin.LIMB_MFMA, id="limb"), pytest.param(spin.VALU, id="valu")]
SHAPES = [(1, 1, 1, 1, 1), (2, 1, 1, 1, 1), (2, 1, 33, 31, 32), (3, 2, 130, 70, 45), (5, 1, 64, 64, 64),
          (8, 1, 40, 40, 40), (2, 3, 17, 200, 100), (3, 1, 129, 260, 257), (1, 1, 128, 128, 32),
          (2, 1, 300, 131, 66), (2, 1, 7, 5, 1001), (3, 5, 128, 128, 64)]


def matmul_case(n, batch, M, N, K, seed, path):
    rng = np.random.default_rng(seed)
    X, Y = rand_ring(rng, (n, batch, M, K)), rand_ring(rng, (n, batch, K, N))
    A, B, C = oracle.dealer_matmul(n, batch, M, N, K, seed=seed, l=32)
    want = oracle.beaver_matmul(X, Y, A, B, C, l=32)
    got = R.beaver_matmul(dev(X), dev(Y), dev(A), dev(B), dev(C), path=path)
    torch.cuda.synchronize()
    return host(got), want, (X, Y)


@pytest.mark.parametrize("path", PATHS)
@pytest.mark.parametrize("n,batch,M,N,K", SHAPES)
def test_beaver_matmul(n, batch, M, N, K, path):
    got, want, (X, Y) = matmul_case(n, batch, M, N, K, n * 7 + M, path)
    assert (got == want).all()
    # reconstruction: the shares sum to the plain ring product
    xs, ys = oracle.open_(X.reshape(n, -1), l=32).reshape(X.shape[1:]), oracle.open_(Y.reshape(n, -1), l=32).reshape(Y.shape[1:])
    for b in range(batch):
        assert ((got.sum(axis=0) & M32)[b] == oracle.ring_matmul(xs[b], ys[b], l=32)).all()


def test_limb_path_worst_case_digits_and_long_inner_dimension():
    # every digit of every operand equal to -128 (value 0x7F7F7F80) with K so long that the int32
    # accumulators wrap many times: 4 digits need at most 32 exact bits per diagonal, so the wrapped
    # sums must still give the exact ring product.
    n, M, N, K = 2, 32, 32, 70000
    worst = np.uint64(0x7F7F7F80)
    X = np.zeros((n, 1, M, K), dtype=np.uint64); X[:] = worst
    Y = np.zeros((n, 1, K, N), dtype=np.uint64); Y[:] = worst
    A = np.zeros_like(X); B = np.zeros_like(Y); A[1] = worst; B[1] = worst
    C = np.zeros((n, 1, M, N), dtype=np.uint64)
    want = oracle.beaver_matmul(X, Y, A, B, C, l=32)
    got = R.beaver_matmul(dev(X), dev(Y), dev(A), dev(B), dev(C), path=spin.LIMB_MFMA)
    assert (host(got) == want).all()
    g, w, _ = matmul_case(2, 1, 40, 36, 40000 + 8, seed=9, path=spin.LIMB_MFMA)
    assert (g == w).all()


def test_paths_agree_on_a_large_shape_and_sampled_rows_match_the_oracle():
    n, M, N, K = 3, 2048, 1024, 1536
    rng = np.random.default_rng(77)
    X, Y = rand_ring(rng, (n, 1, M, K)), rand_ring(rng, (n, 1, K, N))
    A, B, C = oracle.dealer_matmul(n, 1, M, N, K, seed=77, l=32)
    args = [dev(t) for t in (X, Y, A, B, C)]
    zl = R.beaver_matmul(*args, path=spin.LIMB_MFMA)
    zv = R.beaver_matmul(*args, path=spin.VALU)
    assert torch.equal(zl, zv)
    rows = np.sort(rng.choice(M, 64, replace=False)); rows[0], rows[-1] = 0, M - 1
    want = oracle.beaver_matmul(X, Y, A, B, C, l=32, rows=rows)
    assert (host(zl)[:, :, rows] == want).all()


def test_fixed32_pipeline_after_a_local_cast():
    # Fixed64 shares with f = 8 are cast locally, multiplied and truncated in the 32-bit ring; the decoded
    # result is the product to within the two truncation units.
    n, f, count = 3, 8, 50000
    rng = np.random.default_rng(8)
    xr, yr = rng.uniform(-8, 8, count), rng.uniform(-8, 8, count)
    X64 = oracle.share(oracle.encode(xr, f), n, 1, oracle.STREAM_X)
    Y64 = oracle.share(oracle.encode(yr, f), n, 1, oracle.STREAM_Y)
    xd, yd = R.cast_from_64(dev64(X64)), R.cast_from_64(dev64(Y64))
    a, b, c = oracle.dealer_mul(n, count, seed=2, l=32)
    r, rt, rm = oracle.trunc_dealer(n, count, f, seed=3, l=32)
    zd = R.trunc(R.beaver_mul(xd, yd, dev(a), dev(b), dev(c)), dev(r), dev(rt), dev(rm), f)
    zo = oracle.trunc(oracle.beaver_mul(oracle.cast_64_to_32(X64), oracle.cast_64_to_32(Y64), a, b, c, l=32),
                      r, rt, rm, f, l=32)
    assert (host(zd) == zo).all()
    got = oracle.decode(host(R.open(zd)), f, l=32)
    assert np.abs(got - xr * yr).max() <= 2.0 ** -f * (1 + 2) * 8
