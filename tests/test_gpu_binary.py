"""GPU-vs-oracle parity of the binary-sharing kernels (packed XOR sharing, XOR open, AND with bit triples)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2402_02320_amd import spin

pytestmark = pytest.mark.gpu


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int64)).cuda()


def host(t):
    return t.cpu().numpy().view(np.uint64)


@pytest.mark.parametrize("n", [1, 2, 3, 4, 5, 6, 7, 8])
@pytest.mark.parametrize("count", [1, 2, 999, 65536 + 3])
def test_binary_share_open_and(n, count):
    rng = np.random.default_rng(100 * n + count)
    x, y = rng.integers(0, 1 << 64, size=(2, count), dtype=np.uint64)
    xs, ys = oracle.bshare(x, n, 3, 1), oracle.bshare(y, n, 3, 2)
    xd = spin.bshare(dev(x), n, 3, 1)
    assert (host(xd) == xs).all()
    assert (host(spin.bopen(xd)) == x).all()
    m = rng.integers(0, 1 << 64, size=(n, count), dtype=np.uint64)
    assert (host(spin.bopen(xd, dev(m))) == oracle.bopen(xs, m)).all()
    a, b, c = oracle.dealer_and(n, count, seed=3)
    want = oracle.beaver_and(xs, ys, a, b, c)
    zd = spin.beaver_and(xd, dev(ys), dev(a), dev(b), dev(c))
    assert (host(zd) == want).all()
    assert (host(spin.bopen(zd)) == (x & y)).all()
    spin.beaver_and(xd, dev(ys), dev(a), dev(b), dev(c), out=xd)        # in place
    assert (host(xd) == want).all()


def test_binary_and_at_config2_vector_length():
    n, count = 2, 1 << 24
    rng = np.random.default_rng(5)
    x, y = rng.integers(0, 1 << 64, size=(2, count), dtype=np.uint64)
    xs, ys = oracle.bshare(x, n, 4, 1), oracle.bshare(y, n, 4, 2)
    a, b, c = oracle.dealer_and(n, count, seed=4)
    zd = spin.beaver_and(dev(xs), dev(ys), dev(a), dev(b), dev(c))
    assert (host(zd) == oracle.beaver_and(xs, ys, a, b, c)).all()
    assert (host(spin.bopen(zd)) == (x & y)).all()                       # streaming-size open, plain and masked
    assert (host(spin.bopen(zd, dev(a))) == oracle.bopen(host(zd), a)).all()
