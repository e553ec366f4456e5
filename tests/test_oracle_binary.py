"""Pins of the oracle's binary-sharing functions (Section 4.1 binary sharing; XOR is local, Section 4.3):
exhaustive truth tables over every bit combination and share pattern, and numpy's bitwise operators."""
import itertools

import numpy as np
import pytest

import oracle


@pytest.mark.parametrize("n", [1, 2, 3, 5, 8])
def test_bshare_reconstructs_by_xor(n):
    rng = np.random.default_rng(n)
    x = rng.integers(0, 1 << 64, size=300, dtype=np.uint64)
    sh = oracle.bshare(x, n, 7, oracle.STREAM_X)
    assert (np.bitwise_xor.reduce(sh, axis=0) == x).all()
    for i in range(1, n):
        assert sh[i, 9] == oracle.rand64(7, oracle.STREAM_X, i, 9)
    assert (oracle.bopen(sh) == x).all()
    m = rng.integers(0, 1 << 64, size=(n, 300), dtype=np.uint64)
    assert (oracle.bopen(sh, m) == x ^ np.bitwise_xor.reduce(m, axis=0)).all()


def test_and_triples_are_consistent():
    a, b, c = oracle.dealer_and(3, 500, seed=5)
    av, bv, cv = (np.bitwise_xor.reduce(t, axis=0) for t in (a, b, c))
    assert (cv == av & bv).all()


@pytest.mark.parametrize("n", [2, 3])
def test_beaver_and_truth_table_over_every_share_pattern(n):
    # one bit position per word; every assignment of the 5n share bits (x, y, a, b shares free, c's last share
    # fixed by c = a & b): 2^(5n-1) cases for n = 2, 3
    free = 5 * n - 1
    cases = np.array(list(itertools.product((0, 1), repeat=free)), dtype=np.uint64)
    xs, ys, as_, bs = (cases[:, k * n:(k + 1) * n].T.copy() for k in range(4))
    cpart = cases[:, 4 * n:].T
    av, bv = np.bitwise_xor.reduce(as_, axis=0), np.bitwise_xor.reduce(bs, axis=0)
    c0 = (av & bv) ^ (np.bitwise_xor.reduce(cpart, axis=0) if n > 1 else 0)
    cs = np.concatenate([c0[None], cpart]).astype(np.uint64)
    z = oracle.beaver_and(xs, ys, as_, bs, cs)
    xv, yv = np.bitwise_xor.reduce(xs, axis=0), np.bitwise_xor.reduce(ys, axis=0)
    assert (np.bitwise_xor.reduce(z, axis=0) == (xv & yv)).all()
    assert z.max() <= 1                                         # no bit leaks into other positions


def test_beaver_and_words_against_numpy():
    rng = np.random.default_rng(9)
    n, L = 5, 1000
    x, y = rng.integers(0, 1 << 64, size=(2, L), dtype=np.uint64)
    xs, ys = oracle.bshare(x, n, 3, 1), oracle.bshare(y, n, 3, 2)
    a, b, c = oracle.dealer_and(n, L, seed=3)
    z = oracle.beaver_and(xs, ys, a, b, c)
    assert (np.bitwise_xor.reduce(z, axis=0) == (x & y)).all()
    e = x ^ np.bitwise_xor.reduce(a, axis=0)
    f = y ^ np.bitwise_xor.reduce(b, axis=0)
    for i in range(n):
        want = c[i] ^ (e & b[i]) ^ (a[i] & f) ^ ((e & f) if i == 0 else 0)
        assert (z[i] == want).all()
