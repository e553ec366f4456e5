"""Pins of the 128-bit oracle (oracle/spin_oracle128.c): Python integers for every function, the closed
form of the truncation at l = 128, and agreement of the low 64 bits with the 64-bit oracle where the
mathematics demands it (sums and products mod 2^64 are the low words of those mod 2^128)."""
import numpy as np
import pytest

import oracle
from oracle import r128

M128 = (1 << 128) - 1


def rand_ring(rng, shape):
    return rng.integers(0, 1 << 64, size=tuple(shape) + (2,), dtype=np.uint64)


def signed(v):
    return v - (1 << 128) if v >> 127 else v


def big_matmul(P, Q):
    M, K = P.shape
    N = Q.shape[1]
    return np.array([[sum(int(P[m, k]) * int(Q[k, q]) for k in range(K)) & M128 for q in range(N)]
                     for m in range(M)], dtype=object)


def test_int_conversion_round_trip():
    vals = [0, 1, M128, 1 << 64, (1 << 127) + 5, 0x0123456789ABCDEF_FEDCBA9876543210]
    assert r128.to_ints(r128.from_ints(vals)).tolist() == vals


@pytest.mark.parametrize("n", [1, 2, 3, 5])
def test_share_open(n):
    rng = np.random.default_rng(n)
    x = rand_ring(rng, (50,))
    sh = r128.share(x, n, 7, oracle.STREAM_X)
    total = sum(r128.to_ints(sh[i]) for i in range(n)) & M128
    assert (total == r128.to_ints(x)).all()
    for i in range(1, n):       # a 128-bit generator word is the pair of 64-bit outputs 2k, 2k+1
        assert sh[i, 3, 0] == oracle.rand64(7, oracle.STREAM_X, i, 6)
        assert sh[i, 3, 1] == oracle.rand64(7, oracle.STREAM_X, i, 7)
    assert (r128.open_(sh) == x).all()
    m = rand_ring(rng, (n, 50))
    want = (sum(r128.to_ints(sh[i]) - r128.to_ints(m[i]) for i in range(n))) & M128
    assert (r128.to_ints(r128.open_(sh, m)) == want).all()


def test_ring_matmul_against_integers_and_low_words_against_the_64_bit_oracle():
    rng = np.random.default_rng(5)
    P, Q = rand_ring(rng, (6, 9)), rand_ring(rng, (9, 4))
    got = r128.ring_matmul(P, Q)
    assert (r128.to_ints(got) == big_matmul(r128.to_ints(P), r128.to_ints(Q))).all()
    assert (got[..., 0] == oracle.ring_matmul(P[..., 0], Q[..., 0])).all()


def test_triples_are_consistent():
    n, batch, M, N, K = 3, 2, 4, 3, 5
    A, B, C = r128.dealer_matmul(n, batch, M, N, K, seed=11)
    a, b, c = (sum(r128.to_ints(T[i]) for i in range(n)) & M128 for T in (A, B, C))
    for bb in range(batch):
        assert (c[bb] == big_matmul(a[bb], b[bb])).all()
    ea, eb, ec = r128.dealer_mul(4, 100, seed=12)
    av, bv, cv = (sum(r128.to_ints(t[i]) for i in range(4)) & M128 for t in (ea, eb, ec))
    assert (cv == (av * bv) & M128).all()


@pytest.mark.parametrize("n", [1, 2, 3, 5])
def test_beaver_matmul_reconstructs_and_follows_the_share_formula(n):
    rng = np.random.default_rng(20 + n)
    batch, M, N, K = 2, 5, 4, 6
    x, y = rand_ring(rng, (batch, M, K)), rand_ring(rng, (batch, K, N))
    X, Y = r128.share(x, n, 31, oracle.STREAM_X), r128.share(y, n, 31, oracle.STREAM_Y)
    A, B, C = r128.dealer_matmul(n, batch, M, N, K, seed=31)
    Z = r128.beaver_matmul(X, Y, A, B, C)
    z = sum(r128.to_ints(Z[i]) for i in range(n)) & M128
    xi, yi = r128.to_ints(x), r128.to_ints(y)
    E = (xi - sum(r128.to_ints(A[i]) for i in range(n))) & M128
    F = (yi - sum(r128.to_ints(B[i]) for i in range(n))) & M128
    for bb in range(batch):
        assert (z[bb] == big_matmul(xi[bb], yi[bb])).all()
        for i in range(n):
            want = (r128.to_ints(C[i, bb]) + big_matmul(E[bb], r128.to_ints(B[i, bb]))
                    + big_matmul(r128.to_ints(A[i, bb]), F[bb]) + (big_matmul(E[bb], F[bb]) if i == 0 else 0)) & M128
            assert (r128.to_ints(Z[i, bb]) == want).all()


def test_beaver_mul_against_integers():
    rng = np.random.default_rng(60)
    n, L = 3, 200
    x, y = rand_ring(rng, (L,)), rand_ring(rng, (L,))
    xs, ys = r128.share(x, n, 61, 1), r128.share(y, n, 61, 2)
    a, b, c = r128.dealer_mul(n, L, seed=61)
    z = r128.beaver_mul(xs, ys, a, b, c)
    assert ((sum(r128.to_ints(z[i]) for i in range(n)) & M128) == (r128.to_ints(x) * r128.to_ints(y)) & M128).all()
    e = (r128.to_ints(x) - sum(r128.to_ints(a[i]) for i in range(n))) & M128
    f = (r128.to_ints(y) - sum(r128.to_ints(b[i]) for i in range(n))) & M128
    for i in range(n):
        want = (r128.to_ints(c[i]) + e * r128.to_ints(b[i]) + r128.to_ints(a[i]) * f + (e * f if i == 0 else 0)) & M128
        assert (r128.to_ints(z[i]) == want).all()


@pytest.mark.parametrize("n,f", [(2, 16), (3, 40), (5, 1), (2, 125)])
def test_trunc_closed_form(n, f):
    rng = np.random.default_rng(90 + n + f)
    L = 600
    xs = [int(v) for v in rng.integers(-(1 << 62), 1 << 62, size=L)]
    xs = [x * int(s) for x, s in zip(xs, rng.integers(1, 1 << 62, size=L))]         # up to ~2^124
    xs[:4] = [-(1 << 126), (1 << 126) - 1, 0, -1]
    X = r128.share(r128.from_ints(xs), n, 91, oracle.STREAM_X)
    r, rt, rm = r128.trunc_dealer(n, L, f, seed=91)
    rv, tv, mv = (sum(r128.to_ints(t[i]) for i in range(n)) & M128 for t in (r, rt, rm))
    assert (tv == (rv >> f) % (1 << (127 - f))).all() and (mv == rv >> 127).all()
    out = r128.trunc(X, r, rt, rm, f)
    got = sum(r128.to_ints(out[i]) for i in range(n)) & M128
    for k in range(L):
        v = ((xs[k] + (1 << 126)) % (1 << f)) + (int(rv[k]) % (1 << f)) >= (1 << f)
        assert signed(int(got[k])) == (xs[k] >> f) + v
