"""Pins of the oracle at ring width l = 32 (the Fixed32 representation of Section 7.1).

The oracle is the l-parametrised C code used for l = 64; what fixes it at l = 32 independently of
itself: reduction mod 2^32 is a ring homomorphism Z_2^64 -> Z_2^32, so every linear or multiplicative
step run on 64-bit inputs and then reduced must equal the 32-bit run on the reduced inputs (the
generator word of the narrow ring is the low half of the wide one); Python integers; the closed form of
the truncation; and the paper's two statements about Fixed32: the cast from Fixed64 is local, and
products overflow once the precision exceeds 16 bits.
"""
import numpy as np

import oracle

M32 = np.uint64(0xFFFFFFFF)


def rand_u64(rng, shape):
    return rng.integers(0, 1 << 64, size=shape, dtype=np.uint64)


def test_reduction_mod_2_32_commutes_with_share_open_mul_and_matmul():
    rng = np.random.default_rng(32)
    n, count = 3, 500
    x, y = rand_u64(rng, count), rand_u64(rng, count)
    X64, Y64 = oracle.share(x, n, 5, oracle.STREAM_X), oracle.share(y, n, 5, oracle.STREAM_Y)
    X32, Y32 = oracle.share(x & M32, n, 5, oracle.STREAM_X, l=32), oracle.share(y & M32, n, 5, oracle.STREAM_Y, l=32)
    assert (X64 & M32 == X32).all() and X32.max() <= M32
    assert (oracle.open_(X32, l=32) == x & M32).all()
    a64, b64, c64 = oracle.dealer_mul(n, count, seed=6)
    a32, b32, c32 = oracle.dealer_mul(n, count, seed=6, l=32)
    assert (a64 & M32 == a32).all() and (b64 & M32 == b32).all() and (c64 & M32 == c32).all()
    z64 = oracle.beaver_mul(X64, Y64, a64, b64, c64)
    z32 = oracle.beaver_mul(X32, Y32, a32, b32, c32, l=32)
    assert (z64 & M32 == z32).all()
    assert (oracle.open_(z32, l=32) == (x * y) & M32).all()

    nb, M, N, K = 2, 9, 7, 21
    Xm, Ym = rand_u64(rng, (n, nb, M, K)), rand_u64(rng, (n, nb, K, N))
    A64, B64, C64 = oracle.dealer_matmul(n, nb, M, N, K, seed=8)
    A32, B32, C32 = oracle.dealer_matmul(n, nb, M, N, K, seed=8, l=32)
    assert (C64 & M32 == C32).all()
    Z64 = oracle.beaver_matmul(Xm, Ym, A64, B64, C64)
    Z32 = oracle.beaver_matmul(Xm & M32, Ym & M32, A32, B32, C32, l=32)
    assert (Z64 & M32 == Z32).all()


def test_matmul_and_mul_against_python_integers_mod_2_32():
    rng = np.random.default_rng(33)
    n, M, N, K = 2, 4, 3, 5
    X, Y = rand_u64(rng, (n, 1, M, K)) & M32, rand_u64(rng, (n, 1, K, N)) & M32
    A, B, C = oracle.dealer_matmul(n, 1, M, N, K, seed=3, l=32)
    Z = oracle.beaver_matmul(X, Y, A, B, C, l=32)
    mod = 1 << 32
    xs = [[sum(int(X[i, 0, m, k]) for i in range(n)) % mod for k in range(K)] for m in range(M)]
    ys = [[sum(int(Y[i, 0, k, q]) for i in range(n)) % mod for q in range(N)] for k in range(K)]
    for m in range(M):
        for q in range(N):
            want = sum(xs[m][k] * ys[k][q] for k in range(K)) % mod
            assert sum(int(Z[i, 0, m, q]) for i in range(n)) % mod == want
    # the shares themselves, from the update formula in Python integers
    E = [[(xs[m][k] - sum(int(A[i, 0, m, k]) for i in range(n))) % mod for k in range(K)] for m in range(M)]
    F = [[(ys[k][q] - sum(int(B[i, 0, k, q]) for i in range(n))) % mod for q in range(N)] for k in range(K)]
    for i in range(n):
        for m in range(M):
            for q in range(N):
                v = int(C[i, 0, m, q])
                v += sum(E[m][k] * int(B[i, 0, k, q]) + int(A[i, 0, m, k]) * F[k][q] for k in range(K))
                if i == 0:
                    v += sum(E[m][k] * F[k][q] for k in range(K))
                assert v % mod == int(Z[i, 0, m, q])


def test_truncation_closed_form_at_l_32():
    rng = np.random.default_rng(34)
    for n in (2, 3, 5):
        for f in (1, 8, 16, 29):
            count = 4000
            x = rng.integers(-(1 << 30), 1 << 30, size=count, dtype=np.int64)
            x[:2] = (-(1 << 30), (1 << 30) - 1)                    # both ends of the admissible range
            X = oracle.share(x.view(np.uint64) & M32, n, 40 + f, oracle.STREAM_X, l=32)
            r, rt, rm = oracle.trunc_dealer(n, count, f, seed=41 + f, l=32)
            out = oracle.open_(oracle.trunc(X, r, rt, rm, f, l=32), l=32)
            rr = oracle.open_(r, l=32)
            assert (oracle.open_(rt, l=32) == (rr >> np.uint64(f)) & np.uint64((1 << (31 - f)) - 1)).all()
            assert (oracle.open_(rm, l=32) == rr >> np.uint64(31)).all()
            xp = (x + (1 << 30)).astype(np.uint64)
            v = ((xp & np.uint64((1 << f) - 1)) + (rr & np.uint64((1 << f) - 1))) >> np.uint64(f)
            want = ((x >> f) + v.astype(np.int64)).view(np.uint64) & M32
            assert (out == want).all()


def test_local_cast_from_fixed64_keeps_values_that_fit_32_bits():
    # Section 7.1: the cast is performed by each party on its own share, no interaction.
    rng = np.random.default_rng(35)
    n, count = 3, 3000
    x = rng.integers(-(1 << 31), 1 << 31, size=count, dtype=np.int64)
    x[:2] = (-(1 << 31), (1 << 31) - 1)
    X64 = oracle.share(x.view(np.uint64), n, 50, oracle.STREAM_X)
    X32 = oracle.cast_64_to_32(X64)
    assert X32.max() <= M32
    got = oracle.open_(X32, l=32)
    assert (oracle.decode(got, 0, l=32) == x.astype(np.float64)).all()
    # a value outside [-2^31, 2^31) comes back reduced mod 2^32
    big = np.array([(1 << 31), -(1 << 31) - 1, 5 << 40], dtype=np.int64)
    B32 = oracle.cast_64_to_32(oracle.share(big.view(np.uint64), n, 51, oracle.STREAM_X))
    back = oracle.decode(oracle.open_(B32, l=32), 0, l=32)
    assert (back == np.array([-(1 << 31), (1 << 31) - 1, 0], dtype=np.float64)).all()


def test_fixed32_products_overflow_beyond_16_bits_of_precision():
    # Section 7.1: a multiplication doubles the precision, so at l = 32 a product of values of
    # magnitude about 1 survives with f = 8 (2f = 16 bits + integer part) and wraps with f = 16.
    n = 3
    xr = np.array([1.5, -2.25, 3.0, 0.75])
    yr = np.array([1.5, 2.0, -3.0, 4.0])
    for f, survives in ((8, True), (16, False)):
        X = oracle.share(oracle.encode(xr, f, l=32), n, 60, oracle.STREAM_X, l=32)
        Y = oracle.share(oracle.encode(yr, f, l=32), n, 60, oracle.STREAM_Y, l=32)
        a, b, c = oracle.dealer_mul(n, xr.size, seed=61, l=32)
        z = oracle.open_(oracle.beaver_mul(X, Y, a, b, c, l=32), l=32)
        got = oracle.decode(z, 2 * f, l=32)
        assert (got == xr * yr).all() == survives
